// Matrix-core decode attention: the merge kernel and the table of the variants instantiated for the measured
// configurations; decode_mfma_kernel.h holds the kernel itself, decode_mfma_generic_*.hip the wider tables.
#define MIXKVQ_MFMA_MAIN_TU
#include "decode_mfma_generic.h"

namespace mixkvq {

// ---------------------------------------------------------------------------
// Log-sum-exp merge of the partials of one pair (one workgroup per pair):
// m* = max m_i, l* = sum l_i e^(m_i - m*), O = sum O_i e^(m_i - m*) / l*.
// A launch of its own: the kernel boundary makes the partials visible across the chip's L2 slices.  (Merging
// in the attention kernel by the last workgroup of a pair to arrive was measured slower: with agent-scope
// stores, counter and loads the chain store-acknowledge -> atomic -> loads costs more than this launch, and
// device-wide fences cost far more.)
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
decode_merge_pair_kernel(CacheView cv, const float* __restrict__ part, int n_parts, __half* __restrict__ out,
                         float* __restrict__ lse) {
  __shared__ __align__(16) unsigned char smem[kMergeLds];
  const int p = blockIdx.x, tid = threadIdx.x, g = cv.g;
  const int b = p / cv.cfg.Hkv, j = p % cv.cfg.Hkv;
  const size_t stride = (size_t)g * kPartStrideM;
  const float* pbase = part + (size_t)p * n_parts * g * kPartStrideM;
  float* sW = reinterpret_cast<float*>(smem + 64);          // [n_parts][g] weights e^(m_i - m*), m_i first
  float* sML = sW + (kMaxSplits + 1) * 8;                   // [g] m*, then [g] l*
  // Every load of the first 16 parts goes out before anything waits: the (part, head) maxima and sums, and
  // this thread's output channel of up to four heads.
  constexpr int kItems = (kMaxSplits * 8 + 255) / 256;      // (part, head) items per thread
  float my_m[kItems], my_l[kItems];
#pragma unroll
  for (int it = 0; it < kItems; ++it) {
    const int t = tid + 256 * it;
    my_m[it] = -INFINITY;
    my_l[it] = 0.f;
    if (t < n_parts * g) {
      const int sidx = t / g, h = t % g;
      my_m[it] = pbase[sidx * stride + h * kPartStrideM + kD];
      my_l[it] = pbase[sidx * stride + h * kPartStrideM + kD + 1];
    }
  }
  const int d = tid & 127, h0 = tid >> 7;
  float v0[4][16];
#pragma unroll
  for (int hh = 0; hh < 4; ++hh)
#pragma unroll
    for (int i = 0; i < 16; ++i)
      v0[hh][i] = (h0 + 2 * hh < g && i < n_parts) ? pbase[i * stride + (h0 + 2 * hh) * kPartStrideM + d] : 0.f;
#pragma unroll
  for (int it = 0; it < kItems; ++it)
    if (tid + 256 * it < n_parts * g) sW[tid + 256 * it] = my_m[it];
  __syncthreads();
  if (tid < g) {
    float m = -INFINITY;
    for (int s2 = 0; s2 < n_parts; ++s2) m = fmaxf(m, sW[s2 * g + tid]);
    sML[tid] = m;
  }
  __syncthreads();
  float* sLp = sML + 16;                                     // [n_parts][g] weighted l
#pragma unroll
  for (int it = 0; it < kItems; ++it) {
    const int t = tid + 256 * it;
    if (t < n_parts * g) {
      const float wgt = my_m[it] == -INFINITY ? 0.f : __expf(my_m[it] - sML[t % g]);
      sW[t] = wgt;
      sLp[t] = my_l[it] * wgt;
    }
  }
  __syncthreads();
  if (tid < g) {
    float l = 0.f;
    for (int s2 = 0; s2 < n_parts; ++s2) l += sLp[s2 * g + tid];
    sML[8 + tid] = l;
  }
  __syncthreads();
#pragma unroll
  for (int hh = 0; hh < 4; ++hh) {
    const int h = h0 + 2 * hh;
    if (h >= g) break;
    float o = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) o = fmaf(v0[hh][i], i < n_parts ? sW[i * g + h] : 0.f, o);
    for (int s0 = 16; s0 < n_parts; s0 += 16) {
      float v[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = s0 + i < n_parts ? pbase[(s0 + i) * stride + h * kPartStrideM + d] : 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) o = fmaf(v[i], s0 + i < n_parts ? sW[(s0 + i) * g + h] : 0.f, o);
    }
    const size_t bh = (size_t)b * cv.cfg.Hq + (size_t)j * g + h;
    const float lsum = sML[8 + h];
    const float r = lsum > 0.f ? o / lsum : 0.f;      // l == 0: a sequence without tokens
    reinterpret_cast<unsigned short*>(out)[bh * kD + d] =
        cv.cfg.in_dtype ? f32_to_bf16_bits(r) : __half_as_ushort(__float2half_rn(r));
    if (lse && d == 0) lse[bh] = lsum > 0.f ? sML[h] + __logf(lsum) : -INFINITY;
  }
}

hipError_t launch_merge_pair(const CacheView& v, const float* part, int n_splits, __half* out, float* lse, hipStream_t s) {
  decode_merge_pair_kernel<<<dim3(v.P), dim3(256), 0, s>>>(v, part, n_splits, out, lse);
  return hipGetLastError();
}

// Returns true and launches when the configuration is one the matrix-core kernel covers.
bool try_launch_decode_mfma(const CacheView& v, const __half* q, float scale, int n_blocks, int n_res, int n_splits,
                            float* part, __half* out, float* lse, int accumulate_q, NewToken nt, const SeqCounts& sc,
                            hipStream_t s, hipEvent_t ev_start, hipEvent_t ev_stop, hipError_t* err) {
  const mixkvq_config& c = v.cfg;
  // key groups of 32 tokens take the G32 variants, multiples of 64 the others; value groups of 32, 64 or 128 channels
  // records of 32 tokens (one key group each) take the RH variants
  const int rh = c.R == 32 && c.Gk == 32;
  if ((c.R % 64 != 0 && !rh) || (c.Gk % 64 != 0 && c.Gk != 32) || (c.Gv % 64 != 0 && c.Gv != 32) || n_blocks < 1) return false;
  if (v.lay.off_v > kKPartMax || v.lay.rec_bytes - v.lay.off_v_s > kVMetaMax) return false;
  const int nvg = v.lay.NVG;
  const int nkl = (v.lay.off_v / 16 + 63) / 64;
  const int g32 = c.Gk == 32 && !rh;
  const int paged = v.table != nullptr;
  hipError_t e = hipErrorInvalidValue;
  bool ok = true;
#define MIXKVQ_CASE(K4_, K16_, NVG_, NKL_, RG_, THR_, G32_, PG_, RH_)                                               \
  if (c.k4 == K4_ && c.k16 == K16_ && nvg == NVG_ && nkl <= NKL_ && c.policy == THR_ && g32 == G32_ && paged == PG_ && \
      rh == RH_ && (RG_ == 0 || (c.R == 128 && c.Gk == 128 && HalfSplit<K4_, K16_, THR_>::off_klo == v.lay.off_klo &&  \
                                 HalfSplit<K4_, K16_, THR_>::off_k4 == v.lay.off_k4 &&                              \
                                 HalfSplit<K4_, K16_, THR_>::off_k16 == v.lay.off_k16 &&                            \
                                 HalfSplit<K4_, K16_, THR_>::off_v == v.lay.off_v)))                                \
    e = launch_one<K4_, K16_, NVG_, NKL_, RG_, THR_, G32_, PG_, RH_>(v, q, scale, n_blocks, n_res, n_splits, part, out, lse,  \
                                                           accumulate_q, nt, sc, s, ev_start, ev_stop);             \
  else
  MIXKVQ_CASE(16, 0, 1, 6, 1, 0, 0, 0, 0)
  MIXKVQ_CASE(0, 12, 1, 8, 1, 0, 0, 0, 0)
  MIXKVQ_CASE(8, 0, 1, 6, 1, 0, 0, 0, 0)
  MIXKVQ_CASE(16, 0, 1, 6, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(0, 12, 1, 8, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(0, 0, 1, 6, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(8, 0, 1, 6, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(24, 0, 1, 6, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(32, 0, 1, 6, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(16, 0, 2, 6, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(0, 12, 2, 8, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(8, 4, 1, 8, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(0, 32, 1, 12, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(0, 4, 1, 6, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(0, 8, 1, 7, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(0, 16, 1, 8, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(0, 24, 1, 10, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(16, 4, 1, 8, 0, 0, 0, 0, 0)
  MIXKVQ_CASE(16, 8, 1, 8, 0, 0, 0, 0, 0)
  // threshold policy: the capacities of the two side tiers
  MIXKVQ_CASE(16, 8, 1, 8, 0, 1, 0, 0, 0)
  MIXKVQ_CASE(16, 0, 1, 6, 0, 1, 0, 0, 0)
  MIXKVQ_CASE(0, 12, 1, 8, 0, 1, 0, 0, 0)
  MIXKVQ_CASE(8, 4, 1, 8, 0, 1, 0, 0, 0)
  // key groups of 32 tokens
  MIXKVQ_CASE(16, 0, 1, 7, 0, 0, 1, 0, 0)
  MIXKVQ_CASE(8, 0, 1, 7, 0, 0, 1, 0, 0)
  MIXKVQ_CASE(0, 0, 1, 7, 0, 0, 1, 0, 0)
  MIXKVQ_CASE(16, 0, 2, 7, 0, 0, 1, 0, 0)
  MIXKVQ_CASE(16, 0, 1, 8, 0, 1, 1, 0, 0)
  // value groups of 32 channels (with key groups of 32 tokens: the group size of the paper's experiments)
  MIXKVQ_CASE(0, 12, 4, 10, 0, 0, 1, 0, 0)
  MIXKVQ_CASE(0, 8, 4, 10, 0, 0, 1, 0, 0)
  MIXKVQ_CASE(16, 8, 4, 10, 0, 1, 1, 0, 0)
  MIXKVQ_CASE(0, 12, 4, 10, 0, 1, 1, 0, 0)
  MIXKVQ_CASE(8, 4, 4, 10, 0, 0, 1, 0, 0)
  MIXKVQ_CASE(0, 12, 1, 10, 0, 0, 1, 0, 0)
  MIXKVQ_CASE(16, 8, 1, 10, 0, 1, 1, 0, 0)
  MIXKVQ_CASE(0, 12, 1, 10, 0, 1, 1, 0, 0)
  MIXKVQ_CASE(16, 16, 4, 12, 0, 1, 1, 0, 0)
  MIXKVQ_CASE(16, 0, 4, 7, 0, 0, 1, 0, 0)
  MIXKVQ_CASE(8, 0, 4, 7, 0, 0, 1, 0, 0)
  MIXKVQ_CASE(16, 0, 4, 8, 0, 1, 1, 0, 0)
  MIXKVQ_CASE(16, 0, 4, 6, 0, 0, 0, 0, 0)
  // paged layout (block table): the main tiers
  MIXKVQ_CASE(16, 0, 1, 6, 0, 0, 0, 1, 0)
  MIXKVQ_CASE(0, 12, 1, 8, 0, 0, 0, 1, 0)
  MIXKVQ_CASE(8, 0, 1, 6, 0, 0, 0, 1, 0)
  MIXKVQ_CASE(16, 8, 1, 8, 0, 1, 0, 1, 0)
  MIXKVQ_CASE(16, 0, 4, 7, 0, 0, 1, 1, 0)
  MIXKVQ_CASE(16, 8, 4, 10, 0, 1, 1, 1, 0)
  // records of 32 tokens (the shorter residual length of the paper's throughput runs), value groups of 32 or 128 channels
  MIXKVQ_CASE(16, 0, 4, 2, 0, 0, 0, 0, 1)
  MIXKVQ_CASE(8, 0, 4, 2, 0, 0, 0, 0, 1)
  MIXKVQ_CASE(0, 0, 4, 2, 0, 0, 0, 0, 1)
  MIXKVQ_CASE(16, 0, 1, 2, 0, 0, 0, 0, 1)
  MIXKVQ_CASE(8, 4, 4, 2, 0, 0, 0, 0, 1)
  MIXKVQ_CASE(16, 8, 4, 3, 0, 1, 0, 0, 1)
  MIXKVQ_CASE(16, 0, 4, 3, 0, 1, 0, 0, 1)
  ok = false;
#undef MIXKVQ_CASE
  if (!ok) {     // not one of the variants above: the wider tables (they take either layout)
    const GenericArgs a{v, q, scale, n_blocks, n_res, n_splits, part, out, lse, accumulate_q, nt, sc, s, ev_start, ev_stop,
                        nkl, g32, rh};
    return rh ? try_launch_generic_rh(a, err) : (g32 ? try_launch_generic_g32(a, err) : try_launch_generic_plain(a, err));
  }
  *err = e;
  return true;
}

}  // namespace mixkvq

#ifdef MIXKVQ_PHASE_CLOCKS
extern "C" int mixkvq_debug_phase_clocks(void* host_dst, size_t bytes) {
  (void)hipDeviceSynchronize();
  return (int)hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(mixkvq::g_phase_clock), bytes);
}
#endif
