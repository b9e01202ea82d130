// Host-side helpers of the C ABI: argument validation shared by the entry
// points, arena sizing, status strings.  Nothing here touches the GPU.
#include "zc_common.hpp"

using namespace zc;

static bool bits_ok(int b) { return b == 2 || b == 4 || b == 8; }

extern "C" size_t zc_arena_bytes(int64_t B, int64_t H, int64_t D, int64_t cap, int32_t bits) {
  if (B <= 0 || H <= 0 || D <= 0 || cap <= 0 || bits <= 0) return 0;
  return (size_t)B * H * cap * D * bits / 8;
}

extern "C" int64_t zc_arena_slots(int64_t n_tokens, int64_t n_chunks) {
  if (n_tokens < 0 || n_chunks < 0) return 0;
  // every chunk may waste up to ZC_SLOT_ALIGN - 1 slots
  return align_up64(n_tokens + n_chunks * (ZC_SLOT_ALIGN - 1), ZC_SLOT_ALIGN);
}

int zc_validate_tensor(const zc_tensor4* t) {
  if (!t || !t->ptr) return ZC_ERR_INVALID_ARG;
  if (t->dtype != ZC_F32 && t->dtype != ZC_F16 && t->dtype != ZC_BF16) return ZC_ERR_UNSUPPORTED;
  if (t->B <= 0 || t->H <= 0 || t->L < 0 || t->D <= 0) return ZC_ERR_INVALID_ARG;
  if (t->D != 64 && t->D != 128) return ZC_ERR_UNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(t->ptr) & 15) return ZC_ERR_INVALID_ARG;
  if ((t->sB & 7) || (t->sH & 7) || (t->sL & 7) || t->sL < t->D) return ZC_ERR_INVALID_ARG;
  return ZC_OK;
}

int zc_validate_packed(const zc_packed* p, bool for_append) {
  if (!p) return ZC_ERR_INVALID_ARG;
  if (p->layout != ZC_LAYOUT_ROW && p->layout != ZC_LAYOUT_TGROUP) return ZC_ERR_UNSUPPORTED;
  if (p->scheme < ZC_SCHEME_CHANNEL || p->scheme > ZC_SCHEME_TOKEN) return ZC_ERR_UNSUPPORTED;
  if (!bits_ok(p->bits_hi) || !bits_ok(p->bits_lo)) return ZC_ERR_UNSUPPORTED;
  if (p->B <= 0 || p->H <= 0) return ZC_ERR_INVALID_ARG;
  if (p->D != 64 && p->D != 128) return ZC_ERR_UNSUPPORTED;
  if (p->cap_hi < 0 || p->cap_lo < 0 || (p->cap_hi % ZC_SLOT_ALIGN) || (p->cap_lo % ZC_SLOT_ALIGN)) return ZC_ERR_INVALID_ARG;
  if (p->n_hi < 0 || p->n_lo < 0 || p->n_hi > p->cap_hi || p->n_lo > p->cap_lo) return ZC_ERR_INVALID_ARG;
  if ((p->n_hi % ZC_SLOT_ALIGN) || (p->n_lo % ZC_SLOT_ALIGN)) return ZC_ERR_INVALID_ARG;
  if (p->max_chunks <= 0 || p->n_chunks < 0 || p->n_chunks > p->max_chunks) return ZC_ERR_INVALID_ARG;
  if ((p->cap_hi > 0 && !p->codes_hi) || (p->cap_lo > 0 && !p->codes_lo)) return ZC_ERR_INVALID_ARG;
  if (!p->chan_scale || !p->chan_zero || !p->chunk_table || !p->chunk_table_host) return ZC_ERR_INVALID_ARG;
  if (p->scheme != ZC_SCHEME_CHANNEL) {
    if ((p->cap_hi > 0 && (!p->tok_scale_hi || !p->tok_zero_hi)) ||
        (p->cap_lo > 0 && (!p->tok_scale_lo || !p->tok_zero_lo)))
      return ZC_ERR_INVALID_ARG;
  }
  if ((reinterpret_cast<uintptr_t>(p->codes_hi) & 15) || (reinterpret_cast<uintptr_t>(p->codes_lo) & 15))
    return ZC_ERR_INVALID_ARG;
  if (p->cap_hi > 0x7fffffff || p->cap_lo > 0x7fffffff) return ZC_ERR_INVALID_ARG;
  (void)for_append;
  return ZC_OK;
}


extern "C" const char* zc_status_string(int status) {
  switch (status) {
    case ZC_OK: return "ok";
    case ZC_ERR_INVALID_ARG: return "invalid argument";
    case ZC_ERR_UNSUPPORTED: return "unsupported dtype, head dimension, bit width, scheme or layout";
    case ZC_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case ZC_ERR_CAPACITY: return "packed cache arena or chunk table is full";
    case ZC_ERR_HIP: return "HIP launch failed";
    case ZC_ERR_STATIC_LIMIT: return "problem needs more scratch memory than the library's static buffer holds";
    default: return "unknown status";
  }
}

extern "C" int zc_version(void) { return 1; }
