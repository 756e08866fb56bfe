// Region-mask pipeline (Sec. 3.3.1 stages 2-3, Sec. 3.3.2 Eq. 5): key-frame propagation
// fused with the max-pool projection onto the latent / token grid, and the two box
// dilations that give M_edit and M_see. Byte masks, any non-zero byte is "set",
// outputs are 0/1. Integer work: results are exact.
#include "common.h"

namespace chorus {

constexpr int kProjThreads = 256;
constexpr int kProjWaves = kProjThreads / 64;

// One workgroup per output row (t_o, y_o). Phase 1 ORs every input row of the window
// (kh rows of each distinct key frame the window's frames map to) into a per-column
// byte vector in LDS; phase 2 ORs kw columns per output site.
// VEC: rows are read as 16-byte chunks (Wp % 16 == 0 and the base 16-byte aligned).
template <bool VEC>
__global__ __launch_bounds__(kProjThreads) void mask_project_kernel(const uint8_t* __restrict__ key_masks, int Kf,
                                                                    const int32_t* __restrict__ frame_key, int Tp, int Hp,
                                                                    int Wp, int kt, int kh, int kw, int t_lead, int Ho, int Wo,
                                                                    uint8_t* __restrict__ out) {
  extern __shared__ uint32_t col_any[];  // ceil(Wp / 16) * 4 words, byte c = OR over the window's rows of column c
  const int t_o = blockIdx.x / Ho, y_o = blockIdx.x % Ho;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int words = ((Wp + 15) / 16) * 4;
  for (int i = tid; i < words; i += kProjThreads) col_any[i] = 0;
  __syncthreads();

  int t0, t1;
  if (t_o < t_lead) {
    t0 = t_o;
    t1 = t_o + 1;
  } else {
    t0 = t_lead + (t_o - t_lead) * kt;
    t1 = min(t0 + kt, Tp);
  }
  const int y0 = y_o * kh, y1 = min(y0 + kh, Hp);
  const int rows_per_frame = y1 - y0;
  const size_t plane = (size_t)Hp * Wp;

  int prev_key = -1;
  for (int t = t0; t < t1; ++t) {
    int key = frame_key ? frame_key[t] : t;
    if (key == prev_key) continue;  // same key frame as the previous frame of this window: nothing new
    prev_key = key;
    if (key < 0 || key >= Kf) continue;  // a frame with no key frame contributes nothing
    const uint8_t* frame = key_masks + (size_t)key * plane + (size_t)y0 * Wp;
    if (VEC) {
      const int chunks = Wp >> 4;
      // lanes walk the 16-byte chunks of a row, the waves share the rows
      for (int c = lane; c < chunks; c += 64) {
        u32x4 acc = {0u, 0u, 0u, 0u};
        for (int r = wave; r < rows_per_frame; r += kProjWaves)
          acc |= *reinterpret_cast<const u32x4*>(frame + (size_t)r * Wp + (size_t)c * 16);
#pragma unroll
        for (int k = 0; k < 4; ++k)
          if (acc[k]) atomicOr(&col_any[c * 4 + k], acc[k]);
      }
    } else {
      for (int c = lane; c < Wp; c += 64) {
        uint32_t acc = 0;
        for (int r = wave; r < rows_per_frame; r += kProjWaves) acc |= frame[(size_t)r * Wp + c];
        if (acc) atomicOr(&col_any[c >> 2], 1u << ((c & 3) * 8));
      }
    }
  }
  __syncthreads();
  const uint8_t* cols = reinterpret_cast<const uint8_t*>(col_any);
  uint8_t* orow = out + ((size_t)t_o * Ho + y_o) * Wo;
  for (int x = tid; x < Wo; x += kProjThreads) {
    const int c0 = x * kw, c1 = min(c0 + kw, Wp);
    uint32_t any = 0;
    for (int c = c0; c < c1; ++c) any |= cols[c];
    orow[x] = any ? 1 : 0;
  }
}

// Eq. 5 with box kernels is separable. One workgroup per (frame t, strip of rows): the OR over the time window
// goes into LDS while the rows of the strip (plus r_see rows of halo) are loaded, then a pass along x and a pass
// along y, each for both radii. Sites beyond the grid count as 0.
constexpr int kHierThreads = 256;
constexpr int kHierLdsBytes = 48 * 1024;

__global__ __launch_bounds__(kHierThreads) void mask_hierarchy_lds_kernel(const uint8_t* __restrict__ base, int T, int H, int W,
                                                                          int et, int eh, int ew, int st, int sh, int sw,
                                                                          int strip, int nstrips, uint8_t* __restrict__ edit,
                                                                          uint8_t* __restrict__ see) {
  extern __shared__ uint8_t hier_lds[];
  const int t = blockIdx.x / nstrips, y0 = (blockIdx.x % nstrips) * strip, y1 = min(H, y0 + strip);
  const int ya = max(0, y0 - sh), yb = min(H, y1 + sh);  // rows held in LDS
  const int n_in = (yb - ya) * W;
  uint8_t* S0 = hier_lds;       // OR over the see time window
  uint8_t* E0 = S0 + n_in;      // OR over the edit time window
  uint8_t* S1 = E0 + n_in;      // ... then along x
  uint8_t* E1 = S1 + n_in;
  const int t0 = max(0, t - st), t1 = min(T - 1, t + st);
  const size_t plane = (size_t)H * W;
  for (int i = threadIdx.x; i < n_in; i += kHierThreads) {
    uint32_t s = 0, e = 0;
    const uint8_t* p = base + (size_t)ya * W + i;
    for (int tt = t0; tt <= t1; ++tt) {
      const uint32_t v = p[tt * plane];
      s |= v;
      e |= (abs(tt - t) <= et) ? v : 0u;
    }
    S0[i] = s ? 1 : 0;
    E0[i] = e ? 1 : 0;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < n_in; i += kHierThreads) {
    const int x = i % W, row = i - x;
    const int xa = max(0, x - sw), xb = min(W - 1, x + sw);
    uint32_t s = 0, e = 0;
    for (int xx = xa; xx <= xb; ++xx) s |= S0[row + xx];
    for (int xx = max(0, x - ew); xx <= min(W - 1, x + ew); ++xx) e |= E0[row + xx];
    S1[i] = s;
    E1[i] = e;
  }
  __syncthreads();
  const int n_out = (y1 - y0) * W;
  for (int i = threadIdx.x; i < n_out; i += kHierThreads) {
    const int x = i % W, y = y0 + i / W;
    uint32_t s = 0, e = 0;
    for (int yy = max(ya, y - sh); yy <= min(yb - 1, y + sh); ++yy) s |= S1[(yy - ya) * W + x];
    for (int yy = max(ya, y - eh); yy <= min(yb - 1, y + eh); ++yy) e |= E1[(yy - ya) * W + x];
    const size_t o = (size_t)t * plane + (size_t)y * W + x;
    if (edit) edit[o] = e;
    if (see) see[o] = s;
  }
}

// Fallback for planes too wide for the LDS kernel. One thread per site: scans the (2 r_see + 1)^3 box once;
// the inner (2 r_edit + 1)^3 box feeds M_edit. Sites beyond the grid count as 0 (the box is cut at the border).
__global__ __launch_bounds__(256) void mask_hierarchy_kernel(const uint8_t* __restrict__ base, int T, int H, int W, int et,
                                                             int eh, int ew, int st, int sh, int sw,
                                                             uint8_t* __restrict__ edit, uint8_t* __restrict__ see) {
  const int n = T * H * W;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const int x = i % W, y = (i / W) % H, t = i / (W * H);
  const int x0 = max(0, x - sw), x1 = min(W - 1, x + sw);
  const int y0 = max(0, y - sh), y1 = min(H - 1, y + sh);
  const int t0 = max(0, t - st), t1 = min(T - 1, t + st);
  uint32_t any_see = 0, any_edit = 0;
  for (int tt = t0; tt <= t1; ++tt) {
    const bool in_t = abs(tt - t) <= et;
    for (int yy = y0; yy <= y1; ++yy) {
      const bool in_ty = in_t && abs(yy - y) <= eh;
      const uint8_t* row = base + ((size_t)tt * H + yy) * W;
      uint32_t row_see = 0, row_edit = 0;
      for (int xx = x0; xx <= x1; ++xx) {
        uint32_t v = row[xx];
        row_see |= v;
        row_edit |= (abs(xx - x) <= ew) ? v : 0u;
      }
      any_see |= row_see;
      any_edit |= in_ty ? row_edit : 0u;
    }
  }
  if (edit) edit[i] = any_edit ? 1 : 0;
  if (see) see[i] = any_see ? 1 : 0;
}

}  // namespace chorus

using namespace chorus;

extern "C" {

int32_t chorus_mask_pooled_extent(int32_t n, int32_t k, int32_t lead) {
  if (k < 1 || lead < 0 || n < lead) return CHORUS_E_ARG;
  return lead + (n - lead + k - 1) / k;
}

int32_t chorus_mask_project(const uint8_t* key_masks, int32_t Kf, const int32_t* frame_key, int32_t Tp, int32_t Hp,
                            int32_t Wp, int32_t kt, int32_t kh, int32_t kw, int32_t t_lead, uint8_t* out, void* stream) {
  if (Kf < 0 || Tp < 0 || Hp < 0 || Wp < 0 || kt < 1 || kh < 1 || kw < 1 || t_lead < 0 || t_lead > Tp) return CHORUS_E_ARG;
  if (!frame_key && Kf != Tp) return CHORUS_E_ARG;
  const int64_t To = t_lead + ((int64_t)Tp - t_lead + kt - 1) / kt;
  const int64_t Ho = ((int64_t)Hp + kh - 1) / kh, Wo = ((int64_t)Wp + kw - 1) / kw;
  if (To * Ho * Wo == 0) return CHORUS_OK;
  if (!key_masks || !out || Kf == 0) return CHORUS_E_ARG;
  if (To * Ho > 0x7fffffffLL || (int64_t)Kf * Hp * Wp > 0x7fffffffffLL) return CHORUS_E_SHAPE;
  const size_t lds = (size_t)((Wp + 15) / 16) * 16;
  if (lds > 64 * 1024) return CHORUS_E_SHAPE;
  hipStream_t s = (hipStream_t)stream;
  const bool vec = (Wp % 16 == 0) && aligned16(key_masks);
  if (vec)
    hipLaunchKernelGGL(mask_project_kernel<true>, dim3((unsigned)(To * Ho)), dim3(kProjThreads), lds, s, key_masks, Kf,
                       frame_key, Tp, Hp, Wp, kt, kh, kw, t_lead, (int)Ho, (int)Wo, out);
  else
    hipLaunchKernelGGL(mask_project_kernel<false>, dim3((unsigned)(To * Ho)), dim3(kProjThreads), lds, s, key_masks, Kf,
                       frame_key, Tp, Hp, Wp, kt, kh, kw, t_lead, (int)Ho, (int)Wo, out);
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

int32_t chorus_mask_hierarchy(const uint8_t* mask_base, int32_t T, int32_t H, int32_t W, const int32_t r_edit[3],
                              const int32_t r_see[3], uint8_t* mask_edit, uint8_t* mask_see, void* stream) {
  if (T < 0 || H < 0 || W < 0 || !r_see) return CHORUS_E_ARG;
  int32_t re[3];
  for (int a = 0; a < 3; ++a) {
    re[a] = r_edit ? r_edit[a] : 0;
    if (re[a] < 0 || r_see[a] < re[a]) return CHORUS_E_ARG;  // Eq. 5 needs r' >= r on every axis
  }
  if (mask_edit && !r_edit) return CHORUS_E_ARG;
  const int64_t n = (int64_t)T * H * W;
  if (n == 0) return CHORUS_OK;
  if (!mask_base || (!mask_edit && !mask_see)) return CHORUS_E_ARG;
  if (mask_base == mask_edit || mask_base == mask_see) return CHORUS_E_ARG;  // every site reads its neighbours
  if (n > 0x7fffffffLL - 256) return CHORUS_E_SHAPE;
  hipStream_t s = (hipStream_t)stream;
  // strips of rows: enough workgroups to spread over the chip, each strip with its r_see halo within the LDS budget
  const int halo = 2 * (r_see[1] < H ? r_see[1] : H);
  const long rows_fit = kHierLdsBytes / (4L * W) - halo;
  if (rows_fit >= 1) {
    int nstrips = (128 + T - 1) / T;
    if (nstrips > H) nstrips = H;
    if (nstrips < 1) nstrips = 1;
    int strip = (H + nstrips - 1) / nstrips;
    if (strip > rows_fit) strip = (int)rows_fit;
    nstrips = (H + strip - 1) / strip;
    const size_t lds = 4 * (size_t)(strip + halo) * W;
    hipLaunchKernelGGL(mask_hierarchy_lds_kernel, dim3((unsigned)((long)T * nstrips)), dim3(kHierThreads), lds, s, mask_base,
                       T, H, W, re[0], re[1], re[2], r_see[0], r_see[1], r_see[2], strip, nstrips, mask_edit, mask_see);
  } else {
    hipLaunchKernelGGL(mask_hierarchy_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, mask_base, T, H, W, re[0],
                       re[1], re[2], r_see[0], r_see[1], r_see[2], mask_edit, mask_see);
  }
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

}  // extern "C"
