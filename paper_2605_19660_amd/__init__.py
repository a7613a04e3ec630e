"""MI355X-native OScaR KV-cache compression + fused decode attention.

``paper_2605_19660_amd.synth``  -- seeded synthetic inputs (no method arithmetic).
``paper_2605_19660_amd.binding`` -- ctypes binding of the C-ABI HIP library (loaded lazily,
fails loudly when the library is missing).
"""
