// Fused softmax / temperature / top-p / seeded draw / log-prob gather: one 1024-thread workgroup per
// row of fp32 logits.  The first pass copies the row into LDS (128 KB at V = 32000, padded by one float per 32 so that
// the per-thread contiguous chunks of the draw passes hit distinct banks) and the later passes read it from there;
// rows that do not fit are re-read from L2 instead.  Sums are kept in double and reduced in a fixed order, so a
// row's result is reproducible bit for bit, and both variants compute the same bits.
#include <math.h>

#include "common.h"
#include "kernels.h"

namespace {

constexpr int ST = 1024;  // threads per row
constexpr int SW = ST / 64;

struct Shared {
  double dred[SW];
  float fred[SW];
  int ired[SW];
  unsigned ured[SW];
  double bcast_d;
  float bcast_f;
  int bcast_i;
  int found;
  int last;
};

__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__device__ double block_sum_d(double v, Shared& sh) {
  v = wave_sum_d(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh.dred[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = 0.0;
#pragma unroll
  for (int i = 0; i < SW; ++i) t += sh.dred[i];
  return t;
}

__device__ unsigned block_sum_u(unsigned v, Shared& sh) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh.ured[threadIdx.x >> 6] = v;
  __syncthreads();
  unsigned t = 0;
#pragma unroll
  for (int i = 0; i < SW; ++i) t += sh.ured[i];
  return t;
}

// max value and the lowest index attaining it
__device__ void block_argmax(float v, int idx, Shared& sh, float& vmax, int& imax) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(v, o);
    int oi = __shfl_xor(idx, o);
    if (ov > v || (ov == v && oi < idx)) { v = ov; idx = oi; }
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { sh.fred[threadIdx.x >> 6] = v; sh.ired[threadIdx.x >> 6] = idx; }
  __syncthreads();
  vmax = sh.fred[0];
  imax = sh.ired[0];
#pragma unroll
  for (int i = 1; i < SW; ++i) {
    float ov = sh.fred[i];
    int oi = sh.ired[i];
    if (ov > vmax || (ov == vmax && oi < imax)) { vmax = ov; imax = oi; }
  }
}

__device__ __forceinline__ uint64_t mix64(uint64_t x) {
  uint64_t z = x + 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Exclusive prefix over the workgroup of one double per thread (thread order), fixed summation order.
__device__ double block_excl_scan_d(double v, Shared& sh, double& total) {
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  double inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    double t = __shfl_up(inc, o);
    if (lane >= o) inc += t;
  }
  __syncthreads();
  if (lane == 63) sh.dred[w] = inc;
  __syncthreads();
  double base = 0.0, tot = 0.0;
#pragma unroll
  for (int i = 0; i < SW; ++i) {
    if (i < w) base += sh.dred[i];
    tot += sh.dred[i];
  }
  total = tot;
  return base + inc - v;
}

__device__ unsigned block_excl_scan_u(unsigned v, Shared& sh) {
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  unsigned inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    unsigned t = __shfl_up(inc, o);
    if (lane >= o) inc += t;
  }
  __syncthreads();
  if (lane == 63) sh.ured[w] = inc;
  __syncthreads();
  unsigned base = 0;
#pragma unroll
  for (int i = 0; i < SW; ++i)
    if (i < w) base += sh.ured[i];
  return base + inc - v;
}

template <bool CACHE>
__global__ __launch_bounds__(ST) void sampler_kernel(const float* __restrict__ logits, int V, SamplerArgs p,
                                                     const SamplerArgs* __restrict__ args_dev,
                                                     const int* step_ptr, int* __restrict__ cur_tok,
                                                     int* adv_seq_len, int* adv_step) {   // (adv_step is step_ptr when set)
  __shared__ Shared sh;
  extern __shared__ float row_s[];   // CACHE: the row, element i at i + i / 32
  if (args_dev) p = *args_dev;       // (uniform: every lane reads the same block)
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const float* grow = logits + (size_t)b * V;
  const int t = step_ptr[b * p.step_stride];
  const size_t out_idx = (size_t)b * p.out_stride + (p.use_step_col ? t : 0);
  int* __restrict__ tok_out = p.tok_out;
  float* __restrict__ lp_out = p.lp_out;
  struct Row {
    const float* g;
    const float* s;
    __device__ __forceinline__ float operator[](int i) const { return CACHE ? s[i + (i >> 5)] : g[i]; }
  } row{grow, row_s};

  // pass 1: raw maximum and its lowest index
  float vloc = -INFINITY;
  int iloc = 0x7fffffff;
  if ((V & 3) == 0) {
    // 16-byte loads, eight in flight per thread: one memory round trip for rows up to 32768 entries instead of a
    // chain of dependent 4-byte loads.  A thread sees its indices in ascending order, so `>` keeps the lowest.
    const int nvec = V >> 2;
    for (int j0 = tid; j0 < nvec; j0 += 8 * ST) {
      float4 q[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) q[u] = *(const float4*)(grow + 4 * (size_t)min(j0 + u * ST, nvec - 1));
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int j = j0 + u * ST;
        if (j < nvec) {
          const float e4[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int i = 4 * j + c;
            if (CACHE) row_s[i + (i >> 5)] = e4[c];
            if (e4[c] > vloc) { vloc = e4[c]; iloc = i; }
          }
        }
      }
    }
  } else {
    for (int i = tid; i < V; i += ST) {
      float v = grow[i];
      if (CACHE) row_s[i + (i >> 5)] = v;
      if (v > vloc) { vloc = v; iloc = i; }
    }
  }
  float vmax;
  int imax;
  block_argmax(vloc, iloc, sh, vmax, imax);

  // pass 2: sums of exp for the raw distribution and for the tempered one
  const float invT = p.greedy ? 1.f : 1.f / p.temperature;
  double sraw = 0.0, stmp = 0.0;
  for (int i = tid; i < V; i += ST) {
    float v = row[i];
    const float eraw = expf(v - vmax);
    sraw += (double)eraw;
    if (!p.greedy) {
      // (v - vmax) * 1.0f is v - vmax exactly, so at temperature 1 the two weights are the same value
      const float e = invT == 1.f ? eraw : expf((v - vmax) * invT);
      stmp += (double)e;
      if (CACHE) row_s[i + (i >> 5)] = e;   // from here on the cached row holds the tempered weights
    }
  }
  // tempered weight of token i: read back from the cache, or recomputed (same expression, same bits)
  auto wgt = [&](int i) -> float { return CACHE ? row_s[i + (i >> 5)] : expf((grow[i] - vmax) * invT); };
  const double Zraw = block_sum_d(sraw, sh);
  // A row of NaNs has no maximum (every comparison is false): the index stays at its start value and is brought
  // into range here, so that whatever follows reads and feeds back a valid token id.
  imax = min(max(imax, 0), V - 1);
  if (p.greedy) {
    if (tid == 0) {
      tok_out[out_idx] = imax;
      lp_out[out_idx] = (float)(-log(Zraw));
      cur_tok[b] = imax;
      if (adv_seq_len) {   // the step's bookkeeping: one more cached token, next response index (every thread read t long ago)
        adv_seq_len[b] += 1;
        adv_step[b] = t + 1;
      }
    }
    return;
  }
  const double Z = block_sum_d(stmp, sh);

  // nucleus: threshold tau = smallest member's weight e = exp((v - vmax)/T); members are e > tau plus the
  // first `ktie` (by index) of those with e == tau.  Found by a bitwise search on the float pattern of tau:
  // the largest tau whose tail mass sum(e >= tau) still reaches top_p * Z.
  float tau = 0.f;
  unsigned ktie = 0xffffffffu;  // all ties kept
  double Zn = Z;
  const bool truncated = p.top_p < 1.f;
  if (truncated) {
    const double need = (double)p.top_p * Z;
    unsigned lo = 0u, hi = 0x3f800000u;  // weights lie in (0, 1]; 1.0f always satisfies need <= ... only if mass(1.0) >= need
    // invariant: mass_ge(lo) >= need.  Search the largest bit pattern with that property.
    while (lo < hi) {
      unsigned mid = lo + ((hi - lo + 1u) >> 1);
      float fm = __uint_as_float(mid);
      double part = 0.0;
      for (int i = tid; i < V; i += ST) {
        float e = wgt(i);
        if (e >= fm) part += (double)e;
      }
      double mass = block_sum_d(part, sh);
      if (mass >= need) lo = mid; else hi = mid - 1u;
    }
    tau = __uint_as_float(lo);
    double pgt = 0.0;
    unsigned ceq = 0;
    for (int i = tid; i < V; i += ST) {
      float e = wgt(i);
      if (e > tau) pgt += (double)e;
      else if (e == tau) ceq++;
    }
    double mass_gt = block_sum_d(pgt, sh);
    unsigned count_eq = block_sum_u(ceq, sh);
    // smallest k >= 1 with mass_gt + k * tau >= need
    unsigned k = 1;
    while (k < count_eq && mass_gt + (double)k * (double)tau < need) ++k;
    ktie = (k >= count_eq) ? 0xffffffffu : k;
    Zn = mass_gt + (double)(ktie == 0xffffffffu ? count_eq : k) * (double)tau;
  }

  // draw: contiguous chunk of indices per thread, exclusive prefix of member weights, first crossing wins
  const int chunk = (V + ST - 1) / ST;
  const int i0 = tid * chunk, i1 = min(V, i0 + chunk);
  unsigned tie_before = 0;
  if (ktie != 0xffffffffu) {
    unsigned c = 0;
    for (int i = i0; i < i1; ++i)
      if (wgt(i) == tau) c++;
    tie_before = block_excl_scan_u(c, sh);
  }
  double local = 0.0;
  {
    unsigned tr = tie_before;
    for (int i = i0; i < i1; ++i) {
      float e = wgt(i);
      bool mem = !truncated || e > tau || (e == tau && (ktie == 0xffffffffu || tr < ktie));
      if (e == tau) tr++;
      if (mem) local += (double)e;
    }
  }
  double total;
  double excl = block_excl_scan_d(local, sh, total);
  const uint64_t key = p.seed ^ ((uint64_t)(b + p.row0) * 0x9E3779B97F4A7C15ull) ^ ((uint64_t)t * 0xBF58476D1CE4E5B9ull);
  const double u = (double)(mix64(key) >> 40) * (1.0 / 16777216.0);
  const double target = u * total;
  if (tid == 0) { sh.found = 0x7fffffff; sh.last = -1; }
  __syncthreads();
  {
    unsigned tr = tie_before;
    double run = excl;
    int mylast = -1;
    bool done = false;
    for (int i = i0; i < i1; ++i) {
      float e = wgt(i);
      bool mem = !truncated || e > tau || (e == tau && (ktie == 0xffffffffu || tr < ktie));
      if (e == tau) tr++;
      if (mem) {
        mylast = i;
        run += (double)e;
        if (!done && run > target) { atomicMin(&sh.found, i); done = true; }
      }
    }
    if (mylast >= 0) atomicMax(&sh.last, mylast);
  }
  __syncthreads();
  if (tid == 0) {
    int tok = sh.found != 0x7fffffff ? sh.found : sh.last;
    if (tok < 0) tok = imax;   // no nucleus member at all (NaN logits): fall back to the arg-max index, which is in range
    float v = grow[tok];
    float lp;
    if (p.logprob_mode == 0)
      lp = (float)((double)(v - vmax) - log(Zraw));
    else
      lp = (float)((double)((v - vmax) * invT) - log(total));
    tok_out[out_idx] = tok;
    lp_out[out_idx] = lp;
    cur_tok[b] = tok;
    if (adv_seq_len) {
      adv_seq_len[b] += 1;
      adv_step[b] = t + 1;
    }
  }
  (void)Zn;
}

// Raw-model log-probability of a given token per row of logits: lp = logit[tok] - max - log(sum exp(logit - max)).
// Row r belongs to flat response slot slot[r]; the token is resp_tokens[slot[r]] and the result goes to out[slot[r]].
__global__ __launch_bounds__(ST) void logprob_gather_kernel(const float* __restrict__ logits, int V,
                                                            const int* __restrict__ slot,
                                                            const int* __restrict__ resp_tokens, float* __restrict__ out,
                                                            int* __restrict__ err_flag) {
  __shared__ Shared sh;
  const int r = blockIdx.x, tid = threadIdx.x;
  const float* row = logits + (size_t)r * V;
  float vloc = -INFINITY;
  int iloc = 0x7fffffff;
  for (int i = tid; i < V; i += ST) {
    float v = row[i];
    if (v > vloc) { vloc = v; iloc = i; }
  }
  float vmax;
  int imax;
  block_argmax(vloc, iloc, sh, vmax, imax);
  double sraw = 0.0;
  for (int i = tid; i < V; i += ST) sraw += (double)expf(row[i] - vmax);
  const double Z = block_sum_d(sraw, sh);
  if (tid == 0) {
    const int sl = slot[r];
    int tok = resp_tokens[sl];
    if (tok < 0 || tok >= V) {
      *err_flag = 1;
      tok = tok < 0 ? 0 : V - 1;
    }
    out[sl] = (float)((double)(row[tok] - vmax) - log(Z));
  }
}

}  // namespace

hipError_t launch_logprob_gather(hipStream_t s, const float* logits, int rows, int V, const int* slot,
                                 const int* resp_tokens, float* out, int* err_flag) {
  if (rows <= 0) return hipSuccess;
  logprob_gather_kernel<<<rows, ST, 0, s>>>(logits, V, slot, resp_tokens, out, err_flag);
  return hipGetLastError();
}

constexpr int SAMPLER_MAX_CACHED_V = 36864;   // 36864 * 33 / 32 floats = 148.5 KB of LDS

hipError_t sampler_configure() {
  return hipFuncSetAttribute((const void*)sampler_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                             (SAMPLER_MAX_CACHED_V + SAMPLER_MAX_CACHED_V / 32) * 4);
}

hipError_t launch_sampler(hipStream_t s, const float* logits, int B, int V, const SamplerArgs& args, const SamplerArgs* args_dev,
                          const int* step_ptr, int* cur_tok, int* advance_seq_len, int* advance_step) {
  if (B <= 0) return hipSuccess;
  if ((advance_seq_len != nullptr) != (advance_step != nullptr)) return hipErrorInvalidValue;
  if (V <= SAMPLER_MAX_CACHED_V)
    sampler_kernel<true><<<B, ST, (size_t)(V + V / 32 + 1) * 4, s>>>(logits, V, args, args_dev, step_ptr, cur_tok, advance_seq_len,
                                                                     advance_step);
  else
    sampler_kernel<false><<<B, ST, 0, s>>>(logits, V, args, args_dev, step_ptr, cur_tok, advance_seq_len, advance_step);
  return hipGetLastError();
}
