// The matrix-core decode kernel for the float zero-point form (zero-point = group minimum,
// x = Delta * c + zero; the quantizer description of the complexity appendix): the same source
// as oscar_decode_mfma.hip with the zero-point form fixed at compile time, as a translation
// unit of its own so that the two sets of variants compile in parallel.
#define OSCAR_MFMA_ZPMIN 1
#include "oscar_decode_mfma.hip"
