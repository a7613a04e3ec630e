// Host-only entry points of the C ABI: validation, sizing, status strings and the
// debug dump that turns the packed page pools back into one code per byte.
#include <string.h>

#include <atomic>
#include <vector>

#include "oscar_common.h"

int oscar_validate_config(const oscar_config* cfg) {
  if (!cfg) return OSCAR_ERR_INVALID_ARG;
  if (cfg->head_dim <= 0 || cfg->n_q_heads <= 0 || cfg->n_kv_heads <= 0 || cfg->bits <= 0 ||
      cfg->k_group <= 0 || cfg->v_group <= 0 || cfg->page_size <= 0)
    return OSCAR_ERR_INVALID_ARG;
  if (cfg->n_q_heads % cfg->n_kv_heads != 0) return OSCAR_ERR_INVALID_ARG;
  if (cfg->page_size % cfg->k_group != 0 || cfg->head_dim % cfg->v_group != 0)
    return OSCAR_ERR_INVALID_ARG;
  if (cfg->io_dtype != OSCAR_F32 && cfg->io_dtype != OSCAR_BF16 && cfg->io_dtype != OSCAR_F16)
    return OSCAR_ERR_INVALID_ARG;
  if (cfg->meta_dtype != OSCAR_F32 && cfg->meta_dtype != OSCAR_F16 &&
      cfg->meta_dtype != OSCAR_BF16)
    return OSCAR_ERR_INVALID_ARG;
  if (cfg->zp_mode != OSCAR_ZP_INT && cfg->zp_mode != OSCAR_ZP_MIN) return OSCAR_ERR_INVALID_ARG;
  if (cfg->norm_scope != OSCAR_NORM_PER_HEAD && cfg->norm_scope != OSCAR_NORM_ALL_KV_HEADS)
    return OSCAR_ERR_INVALID_ARG;
  if (cfg->rotation != OSCAR_ROTATION_ON && cfg->rotation != OSCAR_ROTATION_OFF)
    return OSCAR_ERR_INVALID_ARG;
  if (cfg->scale_mode < OSCAR_SCALE_L2 || cfg->scale_mode > OSCAR_SCALE_MEAN_ABS)
    return OSCAR_ERR_INVALID_ARG;
  // what is built
  if (cfg->head_dim != OSCAR_D || cfg->page_size != OSCAR_R) return OSCAR_ERR_UNSUPPORTED;
  if (cfg->bits != 2 && cfg->bits != 4) return OSCAR_ERR_UNSUPPORTED;
  if (cfg->k_group != 32 && cfg->k_group != 64 && cfg->k_group != 128) return OSCAR_ERR_UNSUPPORTED;
  if (cfg->v_group != 32 && cfg->v_group != 64 && cfg->v_group != 128) return OSCAR_ERR_UNSUPPORTED;
  if (cfg->meta_dtype == OSCAR_BF16) return OSCAR_ERR_UNSUPPORTED;
  if (cfg->norm_scope == OSCAR_NORM_ALL_KV_HEADS && cfg->scale_mode != OSCAR_SCALE_L2)
    return OSCAR_ERR_UNSUPPORTED;
  if (cfg->n_q_heads / cfg->n_kv_heads > OSCAR_MAX_GQA) return OSCAR_ERR_UNSUPPORTED;
  return OSCAR_OK;
}

extern "C" int oscar_version(void) { return OSCAR_VERSION; }

extern "C" const char* oscar_status_string(int status) {
  switch (status) {
    case OSCAR_OK: return "ok";
    case OSCAR_ERR_INVALID_ARG: return "invalid argument";
    case OSCAR_ERR_UNSUPPORTED: return "configuration not built";
    case OSCAR_ERR_CAPACITY: return "sequence would outgrow its block table";
    case OSCAR_ERR_WORKSPACE: return "workspace missing or too small";
    case OSCAR_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

static size_t io_bytes(int dt) { return dt == OSCAR_F32 ? 4 : 2; }

extern "C" int oscar_cache_sizes(const oscar_config* cfg, int32_t batch, int32_t num_pages,
                                 int32_t max_pages_per_seq, oscar_pool_sizes* out) {
  int rc = oscar_validate_config(cfg);
  if (rc != OSCAR_OK) return rc;
  if (!out || batch <= 0 || num_pages <= 0 || max_pages_per_seq <= 0) return OSCAR_ERR_INVALID_ARG;
  const PageGeom g = make_geom(cfg->bits, cfg->k_group, cfg->v_group, cfg->meta_dtype);
  const size_t units = (size_t)num_pages * cfg->n_kv_heads;
  const size_t streams = (size_t)batch * cfg->n_kv_heads;
  out->k_codes = units * g.k_codes_bytes;
  out->k_meta = units * g.k_meta_bytes;
  out->k_norms = units * g.k_norms_bytes;
  out->v_codes = units * g.v_codes_bytes;
  out->v_meta = units * g.v_meta_bytes;
  out->res_k = streams * OSCAR_R * OSCAR_D * 2;
  out->res_v = streams * OSCAR_R * OSCAR_D * io_bytes(cfg->io_dtype);
  out->res_norm = streams * OSCAR_R * g.meta_bytes;
  out->block_table = (size_t)batch * max_pages_per_seq * sizeof(int32_t);
  out->seq_lens = (size_t)batch * sizeof(int32_t);
  out->res_lens = (size_t)batch * sizeof(int32_t);
  out->tickets = sizeof(int32_t);
  out->page_bytes_per_kv_head = (size_t)g.total();
  out->bytes_per_token_kv_head = (size_t)g.total() / OSCAR_R;
  return OSCAR_OK;
}

extern "C" int oscar_cache_layer(const oscar_cache* all_layers, int32_t n_layers, int32_t layer,
                                 oscar_cache* layer_cache) {
  if (!all_layers || !layer_cache || n_layers < 1 || layer < 0 || layer >= n_layers)
    return OSCAR_ERR_INVALID_ARG;
  oscar_pool_sizes sz;
  const int rc = oscar_cache_sizes(&all_layers->cfg, all_layers->batch, all_layers->num_pages,
                                   all_layers->max_pages_per_seq, &sz);
  if (rc != OSCAR_OK) return rc;
  auto slice = [layer](void* base, size_t bytes) -> void* {
    return base ? static_cast<void*>(static_cast<uint8_t*>(base) + (size_t)layer * bytes) : nullptr;
  };
  oscar_cache c = *all_layers;
  c.k_codes = slice(all_layers->k_codes, sz.k_codes);
  c.k_meta = slice(all_layers->k_meta, sz.k_meta);
  c.k_norms = slice(all_layers->k_norms, sz.k_norms);
  c.v_codes = slice(all_layers->v_codes, sz.v_codes);
  c.v_meta = slice(all_layers->v_meta, sz.v_meta);
  c.res_k = slice(all_layers->res_k, sz.res_k);
  c.res_v = slice(all_layers->res_v, sz.res_v);
  c.res_norm = slice(all_layers->res_norm, sz.res_norm);
  c.seq_lens = static_cast<int32_t*>(slice(all_layers->seq_lens, sz.seq_lens));
  c.res_lens = static_cast<int32_t*>(slice(all_layers->res_lens, sz.res_lens));
  c.tickets = static_cast<int32_t*>(slice(all_layers->tickets, sz.tickets));
  *layer_cache = c;   // block_table and dev_status stay shared
  return OSCAR_OK;
}

extern "C" size_t oscar_decode_workspace_bytes(const oscar_config* cfg, int32_t batch,
                                               int32_t num_splits) {
  if (!cfg || batch <= 0 || num_splits <= 0 || cfg->n_q_heads <= 0 || cfg->head_dim <= 0) return 0;
  // per (batch, q head, split): head_dim partial outputs + running max + running sum, fp32
  return (size_t)batch * cfg->n_q_heads * num_splits * (cfg->head_dim + 2) * sizeof(float);
}

// Compute units of the current device, asked of the runtime once per device and process
// (the attribute query is far cheaper than a full property read, and a decode step must not
// pay either on every call).  256 (one MI355X) if the runtime cannot tell.
static int compute_units_of_current_device() {
  constexpr int kMaxDev = 64;
  static std::atomic<int> cached[kMaxDev];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) {
    (void)hipGetLastError();
    return 256;
  }
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n > 0) return n;
  int v = 0;
  if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) {
    (void)hipGetLastError();
    v = 256;
  }
  cached[dev].store(v, std::memory_order_relaxed);
  return v;
}

extern "C" int32_t oscar_decode_auto_splits(const oscar_config* cfg, int32_t batch,
                                            int32_t max_seq_len) {
  if (!cfg || batch <= 0 || cfg->n_kv_heads <= 0) return 1;
  const int n_cu = compute_units_of_current_device();
  const int pages = max_seq_len > 0 ? (max_seq_len + OSCAR_R - 1) / OSCAR_R : 1;
  const int units = batch * cfg->n_kv_heads;
  // two workgroups (8 waves) per CU are resident at a time (one for the register-hungry
  // variants, see oscar_decode_mfma_wgs_per_cu) and every wave wants at least two pages: aim
  // at one round of workgroups
  const int gq = cfg->n_kv_heads > 0 ? cfg->n_q_heads / cfg->n_kv_heads : 1;
  const int ngk = cfg->k_group > 0 ? OSCAR_R / cfg->k_group : 1;
  const int ngv = cfg->v_group > 0 ? OSCAR_D / cfg->v_group : 1;
  const int resident = oscar_decode_mfma_wgs_per_cu(cfg->bits, gq > 4 ? 2 : 1, ngk, ngv);
  int splits = (resident * n_cu) / units;
  const int max_by_pages = pages / 8 > 0 ? pages / 8 : 1;
  if (splits > max_by_pages) splits = max_by_pages;
  if (splits < 1) splits = 1;
  if (splits > 512) splits = 512;
  return splits;
}

namespace {
float meta_at(const std::vector<uint8_t>& buf, size_t idx, int meta_dtype) {
  if (meta_dtype == OSCAR_F32) {
    float f;
    memcpy(&f, buf.data() + idx * 4, 4);
    return f;
  }
  uint16_t h;
  memcpy(&h, buf.data() + idx * 2, 2);
  // fp16 -> fp32 on the host
  const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
  const uint32_t e = (h >> 10) & 0x1fu, m = h & 0x3ffu;
  uint32_t bits;
  if (e == 0) {
    if (m == 0) {
      bits = sign;
    } else {
      int sh = 0;
      uint32_t mm = m;
      while (!(mm & 0x400u)) { mm <<= 1; ++sh; }
      bits = sign | ((uint32_t)(113 - sh) << 23) | ((mm & 0x3ffu) << 13);
    }
  } else if (e == 31) {
    bits = sign | 0x7f800000u | (m << 13);
  } else {
    bits = sign | ((e + 112) << 23) | (m << 13);
  }
  float f;
  memcpy(&f, &bits, 4);
  return f;
}

float io_at(const std::vector<uint8_t>& buf, size_t idx, int dt) {
  if (dt == OSCAR_F32) {
    float f;
    memcpy(&f, buf.data() + idx * 4, 4);
    return f;
  }
  uint16_t h;
  memcpy(&h, buf.data() + idx * 2, 2);
  if (dt == OSCAR_BF16) {
    uint32_t bits = (uint32_t)h << 16;
    float f;
    memcpy(&f, &bits, 4);
    return f;
  }
  std::vector<uint8_t> tmp(2);
  memcpy(tmp.data(), &h, 2);
  return meta_at(tmp, 0, OSCAR_F16);
}
}  // namespace

static int debug_dump_impl(const oscar_cache* c, int32_t b, int32_t h, int32_t cap_tokens,
                           uint8_t* k_codes, float* k_delta, float* k_zero, float* k_norm,
                           uint8_t* v_codes, float* v_delta, float* v_zero, float* res_k,
                           float* res_v, float* res_norm, int32_t* lens, void* stream) {
  if (!c) return OSCAR_ERR_INVALID_ARG;
  int rc = oscar_validate_config(&c->cfg);
  if (rc != OSCAR_OK) return rc;
  if (b < 0 || b >= c->batch || h < 0 || h >= c->cfg.n_kv_heads || cap_tokens < 0)
    return OSCAR_ERR_INVALID_ARG;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  OSCAR_HIP_CHECK(hipStreamSynchronize(st));
  int32_t seq_len = 0, res_len = 0;
  OSCAR_HIP_CHECK(hipMemcpy(&seq_len, c->seq_lens + b, 4, hipMemcpyDeviceToHost));
  OSCAR_HIP_CHECK(hipMemcpy(&res_len, c->res_lens + b, 4, hipMemcpyDeviceToHost));
  if (lens) {
    lens[0] = seq_len;
    lens[1] = res_len;
  }
  const PageGeom g = make_geom(c->cfg.bits, c->cfg.k_group, c->cfg.v_group, c->cfg.meta_dtype);
  const int D = OSCAR_D, R = OSCAR_R, bits = g.bits, Hkv = c->cfg.n_kv_heads;
  const int n_pages = (seq_len - res_len) / R;
  if (n_pages * R > cap_tokens || n_pages > c->max_pages_per_seq) return OSCAR_ERR_CAPACITY;
  std::vector<int32_t> table((size_t)(n_pages > 0 ? n_pages : 1));
  if (n_pages > 0)
    OSCAR_HIP_CHECK(hipMemcpy(table.data(), c->block_table + (size_t)b * c->max_pages_per_seq,
                              (size_t)n_pages * 4, hipMemcpyDeviceToHost));
  std::vector<uint8_t> kc(g.k_codes_bytes), km(g.k_meta_bytes), kn(g.k_norms_bytes),
      vc(g.v_codes_bytes), vm(g.v_meta_bytes);
  const uint32_t mask = (1u << bits) - 1u;
  for (int p = 0; p < n_pages; ++p) {
    const int phys = table[p];
    if (phys < 0 || phys >= c->num_pages) return OSCAR_ERR_INVALID_ARG;
    const size_t pg = (size_t)phys * Hkv + h;
    OSCAR_HIP_CHECK(hipMemcpy(kc.data(), (const uint8_t*)c->k_codes + pg * g.k_codes_bytes, kc.size(), hipMemcpyDeviceToHost));
    OSCAR_HIP_CHECK(hipMemcpy(km.data(), (const uint8_t*)c->k_meta + pg * g.k_meta_bytes, km.size(), hipMemcpyDeviceToHost));
    OSCAR_HIP_CHECK(hipMemcpy(kn.data(), (const uint8_t*)c->k_norms + pg * g.k_norms_bytes, kn.size(), hipMemcpyDeviceToHost));
    OSCAR_HIP_CHECK(hipMemcpy(vc.data(), (const uint8_t*)c->v_codes + pg * g.v_codes_bytes, vc.size(), hipMemcpyDeviceToHost));
    OSCAR_HIP_CHECK(hipMemcpy(vm.data(), (const uint8_t*)c->v_meta + pg * g.v_meta_bytes, vm.size(), hipMemcpyDeviceToHost));
    for (int t = 0; t < R; ++t) {
      const size_t tok = (size_t)p * R + t;
      const int tpos = tok_meta_pos(t);
      for (int j = 0; j < D; ++j) {
        if (k_codes) {
          // key chunk (tile t/16, n = t%16, q4 = j/32), code number j%32
          const int bit = (j % 32) * bits;
          const size_t off = (size_t)chunk_offset(bits, t / 16, t % 16, j / 32) + bit / 8;
          k_codes[tok * D + j] = (uint8_t)((kc[off] >> (bit % 8)) & mask);
        }
        if (v_codes) {
          // value chunk (tile j/16, n = j%16, q4 = t%4), code number vtok_slot(t)
          const int bit = vtok_slot(bits, t) * bits;
          const size_t off = (size_t)chunk_offset(bits, j / 16, j % 16, vtok_q4(t)) + bit / 8;
          v_codes[tok * D + j] = (uint8_t)((vc[off] >> (bit % 8)) & mask);
        }
      }
      if (k_norm) k_norm[tok] = meta_at(kn, (size_t)tpos, c->cfg.meta_dtype);
      for (int gv = 0; gv < g.ngv; ++gv) {
        if (v_delta) v_delta[tok * g.ngv + gv] = meta_at(vm, (size_t)gv * R + tpos, c->cfg.meta_dtype);
        if (v_zero) v_zero[tok * g.ngv + gv] = meta_at(vm, (size_t)(g.ngv + gv) * R + tpos, c->cfg.meta_dtype);
      }
    }
    for (int gk = 0; gk < g.ngk; ++gk)
      for (int j = 0; j < D; ++j) {
        const size_t row = (size_t)p * g.ngk + gk;
        const int pos = kmeta_pos_of_chan(bits, j);
        if (k_delta) k_delta[row * D + j] = meta_at(km, (size_t)gk * D + pos, c->cfg.meta_dtype);
        if (k_zero) k_zero[row * D + j] = meta_at(km, (size_t)(g.ngk + gk) * D + pos, c->cfg.meta_dtype);
      }
  }
  const size_t sh = ((size_t)b * Hkv + h) * R;
  if (res_k) {
    std::vector<uint8_t> buf((size_t)R * D * 2);
    OSCAR_HIP_CHECK(hipMemcpy(buf.data(), (const uint8_t*)c->res_k + sh * D * 2, buf.size(), hipMemcpyDeviceToHost));
    for (size_t i = 0; i < (size_t)R * D; ++i) res_k[i] = io_at(buf, i, OSCAR_F16);
  }
  if (res_v) {
    const size_t eb = io_bytes(c->cfg.io_dtype);
    std::vector<uint8_t> buf((size_t)R * D * eb);
    OSCAR_HIP_CHECK(hipMemcpy(buf.data(), (const uint8_t*)c->res_v + sh * D * eb, buf.size(), hipMemcpyDeviceToHost));
    for (size_t i = 0; i < (size_t)R * D; ++i) res_v[i] = io_at(buf, i, c->cfg.io_dtype);
  }
  if (res_norm) {
    std::vector<uint8_t> buf((size_t)R * g.meta_bytes);
    OSCAR_HIP_CHECK(hipMemcpy(buf.data(), (const uint8_t*)c->res_norm + sh * g.meta_bytes, buf.size(), hipMemcpyDeviceToHost));
    for (int i = 0; i < R; ++i) res_norm[i] = meta_at(buf, (size_t)i, c->cfg.meta_dtype);
  }
  return OSCAR_OK;
}

// No C++ exception crosses the C boundary: a failed host allocation is reported as a status.
extern "C" int oscar_debug_dump(const oscar_cache* c, int32_t b, int32_t h, int32_t cap_tokens,
                                uint8_t* k_codes, float* k_delta, float* k_zero, float* k_norm,
                                uint8_t* v_codes, float* v_delta, float* v_zero, float* res_k,
                                float* res_v, float* res_norm, int32_t* lens, void* stream) {
  try {
    return debug_dump_impl(c, b, h, cap_tokens, k_codes, k_delta, k_zero, k_norm, v_codes, v_delta,
                           v_zero, res_k, res_v, res_norm, lens, stream);
  } catch (...) {
    return OSCAR_ERR_HIP;
  }
}
