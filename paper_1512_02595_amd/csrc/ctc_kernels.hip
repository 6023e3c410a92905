// HIP kernels of the batched CTC cost + gradient for gfx950 (wave64, CDNA4).
//
// Pipeline of one call (appendix "GPU Implementation of CTC Loss Function"; cost of
// Section 3.3 Eq. (ctc); softmax of Section 3.1):
//   setup     per utterance: links between equal label symbols (replaces the appendix's
//             key-value sort: same purpose, one ordered walk per symbol), degenerate costs
//   softmax   per frame row: log2-sum-exp2 of the scaled logits, and the log2 emissions of
//             blank and of every label position, gathered once so that the recursions read
//             them coalesced
//   lattice   alpha and beta recursions, both in one launch on different workgroups
//   gradient  softmax minus the normalised per-symbol occupancy; zero fill of padding
//
// All lattice quantities are base-2 logarithms: v_exp_f32 / v_log_f32 are base 2, so the
// recursion carries no scaling multiplies.  log(0) is represented by kNeg, a large finite
// negative number, which keeps every operation NaN-free: adding emissions to it leaves it
// unchanged, and 2^(kNeg - anything finite) is exactly 0.
//
// alpha and beta are carried and stored in fp64.  Their magnitude grows with the number of
// frames (thousands of bits for a 15 s utterance) while the gradient needs
// alpha + beta - log p to about 1e-5 absolute, which fp32 cannot hold at that magnitude.
// Only the bounded differences that enter exp2/log2 are narrowed to fp32.

#include <hip/hip_runtime.h>

#include "ctc_internal.h"

namespace ctc {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr double kLn2 = 0.6931471805599453;
constexpr double kNeg = -1.0e30;
constexpr int kRowThreads = 256;

__device__ __forceinline__ float fast_exp2(float v) { return __builtin_amdgcn_exp2f(v); }
__device__ __forceinline__ float fast_log2(float v) { return __builtin_amdgcn_logf(v); }

// ---- element access for the two activation types -------------------------------------

struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float load_elem(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_elem(const bf16_t* p, size_t i)
{
    return __uint_as_float(static_cast<uint32_t>(p[i].bits) << 16);
}
__device__ __forceinline__ void store_elem(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ uint16_t to_bf16_bits(float v)
{
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);           // round to nearest, ties to even
    return static_cast<uint16_t>(u >> 16);
}
__device__ __forceinline__ void store_elem(bf16_t* p, size_t i, float v) { p[i].bits = to_bf16_bits(v); }

// ---- workgroup reductions (256 threads = 4 wavefronts), fixed order => repeatable -------

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// `slot` is 4 floats of LDS private to this reduction.
__device__ __forceinline__ float block_sum(float v, float* slot)
{
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) slot[threadIdx.x >> 6] = v;
    __syncthreads();
    return (slot[0] + slot[1]) + (slot[2] + slot[3]);
}
__device__ __forceinline__ float block_max(float v, float* slot)
{
    v = wave_max(v);
    if ((threadIdx.x & 63) == 0) slot[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(slot[0], slot[1]), fmaxf(slot[2], slot[3]));
}

// ---- setup -------------------------------------------------------------------------------
// One workgroup per utterance.  For label position j: the next position holding the same
// symbol (0 = none, else index + 1) in the low 24 bits, and bit 31 set if j is the first
// occurrence of its symbol.  The gradient kernel walks these chains, so the occupancy of a
// symbol is summed in a fixed order (positions ascending) and each symbol has one writer.
__global__ __launch_bounds__(kRowThreads)
void ctc_setup_kernel(const Utt* __restrict__ meta, const int* __restrict__ labels,
                      int* __restrict__ links, float* __restrict__ costs)
{
    const int b = blockIdx.x;
    const Utt m = meta[b];
    const int* lab = labels + m.lab_off;
    for (int j = threadIdx.x; j < m.L; j += kRowThreads) {
        const int c = lab[j];
        int nxt = 0;
        for (int i = j + 1; i < m.L; ++i)
            if (lab[i] == c) { nxt = i + 1; break; }
        bool first = true;
        for (int i = j - 1; i >= 0; --i)
            if (lab[i] == c) { first = false; break; }
        links[m.lab_off + j] = nxt | (first ? static_cast<int>(0x80000000u) : 0);
    }
    if (threadIdx.x == 0 && !(m.flags & kUttRuns)) {
        // No frames: the empty product (cost 0) for an empty label.  Otherwise no alignment.
        costs[b] = (m.Tb == 0 && m.L == 0) ? 0.0f : __builtin_inff();
    }
}

// ---- softmax statistics + emission gather --------------------------------------------------
// One workgroup per valid frame row (t, b).
template <typename T>
__global__ __launch_bounds__(kRowThreads)
void ctc_softmax_kernel(const T* __restrict__ x, const Utt* __restrict__ meta,
                        const int* __restrict__ labels, float* __restrict__ lse,
                        float* __restrict__ emit, int Tt, int B, int A, int blank)
{
    __shared__ float red[8];
    const int t = blockIdx.x, b = blockIdx.y;
    const Utt m = meta[b];
    if (t >= m.Tb) return;
    const T* row = x + (static_cast<size_t>(t) * B + b) * A;

    float mx = -__builtin_inff();
    for (int k = threadIdx.x; k < A; k += kRowThreads) mx = fmaxf(mx, load_elem(row, k));
    mx = block_max(mx, red) * kLog2e;
    float s = 0.0f;
    for (int k = threadIdx.x; k < A; k += kRowThreads)
        s += fast_exp2(fmaf(load_elem(row, k), kLog2e, -mx));
    s = block_sum(s, red + 4);
    const float l2 = mx + fast_log2(s);
    if (threadIdx.x == 0) lse[static_cast<size_t>(b) * Tt + t] = l2;

    if (!(m.flags & kUttRuns)) return;
    const int P = m.L + 1;
    float* erow = emit + m.e_off + static_cast<size_t>(t) * P;
    const int* lab = labels + m.lab_off;
    for (int j = threadIdx.x; j < P; j += kRowThreads) {
        const int sym = (j == 0) ? blank : lab[j - 1];
        erow[j] = fmaf(load_elem(row, sym), kLog2e, -l2);
    }
}

// ---- lattice recursions ------------------------------------------------------------------
// log2(2^a + 2^b) for fp64 a, b with the exponentials taken on the fp32 difference.
__device__ __forceinline__ double lse2(double a, double b)
{
    const double hi = fmax(a, b), lo = fmin(a, b);
    const float d = static_cast<float>(lo - hi);
    return hi + static_cast<double>(fast_log2(1.0f + fast_exp2(d)));
}
__device__ __forceinline__ double lse3(double a, double b, double c)
{
    const double hi = fmax(fmax(a, b), c);
    const float da = static_cast<float>(a - hi), db = static_cast<float>(b - hi),
                dc = static_cast<float>(c - hi);
    // one of the three differences is 0; the other two are the median and the minimum
    const float mid = __builtin_amdgcn_fmed3f(da, db, dc);
    const float mn = fminf(fminf(da, db), dc);
    return hi + static_cast<double>(fast_log2(1.0f + fast_exp2(mid) + fast_exp2(mn)));
}

// Value of lane-1 within the wavefront (DPP wave_shr:1); lane 0 receives `fill`.
__device__ __forceinline__ double from_lower_lane(double v, double fill)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(__double2loint(fill), lo, 0x138, 0xf, 0xf, false);
    hi = __builtin_amdgcn_update_dpp(__double2hiint(fill), hi, 0x138, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}

constexpr int kPrefetch = 8;   // frames of emissions kept in flight ahead of the recursion

// One chain = one direction of one utterance.  Thread j owns the pair
//   forward : (blank state 2j,       label j        = state 2j+1)
//   backward: (blank state 2(L-j),   label L-1-j    = state 2(L-j)-1)
// so that in both directions the only value needed from a neighbour is the label entry of
// pair j-1.  Forward carries alpha including the own frame's emission; backward carries beta
// excluding it (so log alpha + log beta is the log mass of alignments through a state).
//
// Storage (row pitch 2(L+1) doubles, i.e. the appendix's S = 2(L+1) rows with one that stays
// at log 0): alpha_row[s] = alpha(s); beta_row[s+1] = beta(s).
template <bool kBackward>
__device__ __forceinline__ void run_chain(const Utt m, const int u, const int* __restrict__ labels,
                                          const float* __restrict__ emit, double* __restrict__ out,
                                          double* __restrict__ logp, float* __restrict__ costs,
                                          double (*xch)[16])
{
    const int L = m.L, Tb = m.Tb, P = L + 1;
    const int j = threadIdx.x, lane = j & 63, wave = j >> 6;
    const int* lab = labels + m.lab_off;
    const bool has_label = j < L;
    const bool active = j < P;
    const int li = kBackward ? (L - 1 - j) : j;          // label index of this pair's label state
    bool skip = false;                                   // may the label state be entered from pair j-1's label?
    if (has_label && j >= 1) skip = lab[li] != lab[kBackward ? (li + 1) : (li - 1)];

    const float* ebase = emit + m.e_off;
    const int ecol = has_label ? (1 + li) : 0;
    double* obase = out + m.ab_off;
    const int ocol = kBackward ? (2 * (L - j)) : (2 * j);
    const size_t pitch = 2 * static_cast<size_t>(P);

    auto frame_of = [&](int step) { return kBackward ? (Tb - 1 - step) : step; };
    auto store_row = [&](int frame, double blank_v, double label_v) {
        if (!active) return;
        double2 v = kBackward ? make_double2(label_v, blank_v) : make_double2(blank_v, label_v);
        *reinterpret_cast<double2*>(obase + static_cast<size_t>(frame) * pitch + ocol) = v;
    };
    // Exchange: every lane gets the label value of pair j-1 (log 0 for pair 0).
    auto from_prev_pair = [&](double v, int parity) {
        double r = from_lower_lane(v, kNeg);
        if (blockDim.x > 64) {
            if (lane == 63) xch[parity][wave] = v;
            __syncthreads();
            if (lane == 0 && wave > 0) r = xch[parity][wave - 1];
        }
        return r;
    };

    double v_blank, v_label;
    if (!kBackward) {
        const float eb = ebase[0], el = ebase[ecol];
        v_blank = (j == 0) ? static_cast<double>(eb) : kNeg;
        v_label = (j == 0 && has_label) ? static_cast<double>(el) : kNeg;
    } else {
        v_blank = (j == 0) ? 0.0 : kNeg;
        v_label = (j == 0 && has_label) ? 0.0 : kNeg;
    }
    store_row(frame_of(0), v_blank, v_label);

    // Emissions consumed at step s: forward uses frame s, backward uses frame Tb - s (the
    // frame just left).  They do not depend on the recursion, so they are fetched a block of
    // steps ahead.
    auto emission_frame = [&](int step) {
        int f = kBackward ? (Tb - step) : step;
        return min(max(f, 0), Tb - 1);
    };
    float eb_cur[kPrefetch], el_cur[kPrefetch], eb_nxt[kPrefetch], el_nxt[kPrefetch];
#pragma unroll
    for (int i = 0; i < kPrefetch; ++i) {
        const float* r = ebase + static_cast<size_t>(emission_frame(1 + i)) * P;
        eb_cur[i] = r[0];
        el_cur[i] = r[ecol];
    }
    for (int s0 = 1; s0 < Tb; s0 += kPrefetch) {
#pragma unroll
        for (int i = 0; i < kPrefetch; ++i) {
            const float* r = ebase + static_cast<size_t>(emission_frame(s0 + kPrefetch + i)) * P;
            eb_nxt[i] = r[0];
            el_nxt[i] = r[ecol];
        }
#pragma unroll
        for (int i = 0; i < kPrefetch; ++i) {
            const int step = s0 + i;
            if (step < Tb) {
                const double eb = static_cast<double>(eb_cur[i]);
                const double el = static_cast<double>(el_cur[i]);
                double nb, nl;
                if (!kBackward) {
                    const double prev = from_prev_pair(v_label, step & 1);
                    nb = lse2(v_blank, prev) + eb;
                    nl = lse3(v_label, v_blank, skip ? prev : kNeg) + el;
                } else {
                    const double wb = v_blank + eb, wl = v_label + el;
                    const double prev = from_prev_pair(wl, step & 1);
                    nb = lse2(wb, prev);
                    nl = lse3(wl, wb, skip ? prev : kNeg);
                }
                v_blank = active ? nb : kNeg;
                v_label = has_label ? nl : kNeg;
                store_row(frame_of(step), v_blank, v_label);
            }
        }
#pragma unroll
        for (int i = 0; i < kPrefetch; ++i) { eb_cur[i] = eb_nxt[i]; el_cur[i] = el_nxt[i]; }
    }

    if (!kBackward) {
        // p = alpha_{T-1}(2L) + alpha_{T-1}(2L-1): the blank of pair L and the label of pair L-1.
        const double prev = from_prev_pair(v_label, Tb & 1);
        if (j == L) {
            const double lp = lse2(v_blank, prev);
            logp[u] = lp;
            costs[u] = (lp < -1.0e29) ? __builtin_inff() : static_cast<float>(-lp * kLn2);
        }
    }
}

// grid = (utterances whose lattice runs, 2): y = 0 forward, y = 1 backward.
// blockDim.x = 64 * (wavefronts of the longest label); wavefronts beyond an utterance's own
// need only keep the barrier count.
__global__ __launch_bounds__(1024)
void ctc_lattice_kernel(const Utt* __restrict__ meta, const int* __restrict__ order,
                        const int* __restrict__ labels, const float* __restrict__ emit,
                        double* __restrict__ alpha, double* __restrict__ beta,
                        double* __restrict__ logp, float* __restrict__ costs)
{
    __shared__ double xch[2][16];
    const int u = order[blockIdx.x];
    const Utt m = meta[u];
    const int waves_needed = (m.L + 1 + 63) >> 6;
    if (static_cast<int>(threadIdx.x >> 6) >= waves_needed) {
        // Nothing to compute, but keep meeting the barriers of the working wavefronts:
        // one per recursion step, plus the forward chain's final exchange.
        if (blockDim.x > 64) {
            const int barriers = (m.Tb - 1) + (blockIdx.y == 0 ? 1 : 0);
            for (int i = 0; i < barriers; ++i) __syncthreads();
        }
        return;
    }
    if (blockIdx.y == 0)
        run_chain<false>(m, u, labels, emit, alpha, logp, costs, xch);
    else
        run_chain<true>(m, u, labels, emit, beta, logp, costs, xch);
}

// ---- gradient ------------------------------------------------------------------------------
// One workgroup per row (t, b) of the output, padding rows included.
//   gamma_t(s) = 2^(alpha_t(s) + beta_t(s) - log2 p)        mass share of state s
//   grad[k]    = y_t(k) - sum_{s: symbol(s) = k} gamma_t(s) / sum_s gamma_t(s)
// Dividing by the row's own total (equal to 1 up to rounding) keeps every row summing to zero.
template <typename T>
__global__ __launch_bounds__(kRowThreads)
void ctc_gradient_kernel(const T* __restrict__ x, T* __restrict__ grads,
                         const Utt* __restrict__ meta, const int* __restrict__ labels,
                         const int* __restrict__ links, const float* __restrict__ lse,
                         const double* __restrict__ alpha, const double* __restrict__ beta,
                         const double* __restrict__ logp, int Tt, int B, int A, int blank)
{
    __shared__ float red[8];
    __shared__ float g_label[CTC_MAX_LABEL_LENGTH + 1];
    const int t = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const Utt m = meta[b];
    const size_t row_off = (static_cast<size_t>(t) * B + b) * A;
    T* grow = grads + row_off;

    if (t >= m.Tb || !(m.flags & kUttRuns)) {
        for (int k = tid; k < A; k += kRowThreads) store_elem(grow, k, 0.0f);
        return;
    }
    const T* xrow = x + row_off;
    const int L = m.L, P = L + 1;
    const size_t pitch = 2 * static_cast<size_t>(P);
    const double* arow = alpha + m.ab_off + static_cast<size_t>(t) * pitch;
    const double* brow = beta + m.ab_off + static_cast<size_t>(t) * pitch;
    const double lp = logp[b];

    float z = 0.0f, zb = 0.0f;
    for (int j = tid; j < P; j += kRowThreads) {
        const double2 a = *reinterpret_cast<const double2*>(arow + 2 * j);
        const double bb = brow[2 * j + 1], bl = brow[2 * j + 2 < static_cast<int>(pitch) ? 2 * j + 2 : 0];
        const float gb = fast_exp2(static_cast<float>(a.x + bb - lp));
        const float gl = (j < L) ? fast_exp2(static_cast<float>(a.y + bl - lp)) : 0.0f;
        g_label[j] = gl;
        z += gb + gl;
        zb += gb;
    }
    z = block_sum(z, red);
    zb = block_sum(zb, red + 4);
    const float inv_z = 1.0f / z;
    const float l2 = lse[static_cast<size_t>(b) * Tt + t];

    for (int k = tid; k < A; k += kRowThreads)
        store_elem(grow, k, fast_exp2(fmaf(load_elem(xrow, k), kLog2e, -l2)));
    // The symbols that occur in the label are rewritten below by other threads of this
    // workgroup: make the stores above complete before any of those is issued.
    __threadfence_block();
    __syncthreads();

    const int* lab = labels + m.lab_off;
    const int* lnk = links + m.lab_off;
    for (int j = tid; j < L; j += kRowThreads) {
        int link = lnk[j];
        if (link < 0) {                       // first occurrence of its symbol: sum the chain
            float occ = g_label[j];
            int nxt = link & 0xFFFFFF;
            while (nxt) {
                occ += g_label[nxt - 1];
                nxt = lnk[nxt - 1] & 0xFFFFFF;
            }
            const int c = lab[j];
            store_elem(grow, c, fast_exp2(fmaf(load_elem(xrow, c), kLog2e, -l2)) - occ * inv_z);
        }
    }
    if (tid == 0)
        store_elem(grow, blank, fast_exp2(fmaf(load_elem(xrow, blank), kLog2e, -l2)) - zb * inv_z);
}

template <typename F>
int checked_launch(F&& f)
{
    f();
    return static_cast<int>(hipGetLastError());
}

}  // namespace

int launch_setup(const Launch& p, void* stream)
{
    auto* meta = reinterpret_cast<const Utt*>(p.ws + p.lay.meta);
    auto* labels = reinterpret_cast<const int*>(p.ws + p.lay.labels);
    auto* links = reinterpret_cast<int*>(p.ws + p.lay.links);
    return checked_launch([&] {
        hipLaunchKernelGGL(ctc_setup_kernel, dim3(p.B), dim3(kRowThreads), 0,
                           static_cast<hipStream_t>(stream), meta, labels, links, p.costs);
    });
}

int launch_softmax(const Launch& p, void* stream)
{
    auto* meta = reinterpret_cast<const Utt*>(p.ws + p.lay.meta);
    auto* labels = reinterpret_cast<const int*>(p.ws + p.lay.labels);
    auto* lse = reinterpret_cast<float*>(p.ws + p.lay.lse);
    auto* emit = reinterpret_cast<float*>(p.ws + p.lay.emit);
    const dim3 grid(p.T, p.B), block(kRowThreads);
    auto s = static_cast<hipStream_t>(stream);
    return checked_launch([&] {
        if (p.dtype == CTC_DTYPE_F32)
            hipLaunchKernelGGL(ctc_softmax_kernel<float>, grid, block, 0, s,
                               static_cast<const float*>(p.x), meta, labels, lse, emit,
                               p.T, p.B, p.A, p.blank);
        else
            hipLaunchKernelGGL(ctc_softmax_kernel<bf16_t>, grid, block, 0, s,
                               static_cast<const bf16_t*>(p.x), meta, labels, lse, emit,
                               p.T, p.B, p.A, p.blank);
    });
}

int launch_lattice(const Launch& p, void* stream)
{
    if (p.n_run == 0) return 0;
    auto* meta = reinterpret_cast<const Utt*>(p.ws + p.lay.meta);
    auto* order = reinterpret_cast<const int*>(p.ws + p.lay.order);
    auto* labels = reinterpret_cast<const int*>(p.ws + p.lay.labels);
    auto* emit = reinterpret_cast<const float*>(p.ws + p.lay.emit);
    auto* alpha = reinterpret_cast<double*>(p.ws + p.lay.alpha);
    auto* beta = reinterpret_cast<double*>(p.ws + p.lay.beta);
    auto* logp = reinterpret_cast<double*>(p.ws + p.lay.logp);
    return checked_launch([&] {
        hipLaunchKernelGGL(ctc_lattice_kernel, dim3(p.n_run, 2), dim3(64 * p.max_waves), 0,
                           static_cast<hipStream_t>(stream), meta, order, labels, emit, alpha,
                           beta, logp, p.costs);
    });
}

int launch_gradient(const Launch& p, void* stream)
{
    auto* meta = reinterpret_cast<const Utt*>(p.ws + p.lay.meta);
    auto* labels = reinterpret_cast<const int*>(p.ws + p.lay.labels);
    auto* links = reinterpret_cast<const int*>(p.ws + p.lay.links);
    auto* lse = reinterpret_cast<const float*>(p.ws + p.lay.lse);
    auto* alpha = reinterpret_cast<const double*>(p.ws + p.lay.alpha);
    auto* beta = reinterpret_cast<const double*>(p.ws + p.lay.beta);
    auto* logp = reinterpret_cast<const double*>(p.ws + p.lay.logp);
    const dim3 grid(p.T, p.B), block(kRowThreads);
    auto s = static_cast<hipStream_t>(stream);
    return checked_launch([&] {
        if (p.dtype == CTC_DTYPE_F32)
            hipLaunchKernelGGL(ctc_gradient_kernel<float>, grid, block, 0, s,
                               static_cast<const float*>(p.x), static_cast<float*>(p.grads), meta,
                               labels, links, lse, alpha, beta, logp, p.T, p.B, p.A, p.blank);
        else
            hipLaunchKernelGGL(ctc_gradient_kernel<bf16_t>, grid, block, 0, s,
                               static_cast<const bf16_t*>(p.x), static_cast<bf16_t*>(p.grads), meta,
                               labels, links, lse, alpha, beta, logp, p.T, p.B, p.A, p.blank);
    });
}

}  // namespace ctc
