// HIP kernels of the batched CTC cost + gradient for gfx950 (wave64, CDNA4).
//
// Pipeline of one call (appendix "GPU Implementation of CTC Loss Function"; cost of
// Section 3.3 Eq. (ctc); softmax of Section 3.1; most probable alignment of Section 5.1):
//   upload    the per-call metadata from pinned host memory into the workspace
//             (or plan: the same records built on the GPU from device-resident lengths and labels)
//   setup     per utterance: label positions grouped by symbol (the appendix's one-off
//             key-value sort, done by counting), degenerate costs; rides in the softmax launch
//   softmax   per frame row: log2-sum-exp2 of the scaled logits, and the emissions (softmax
//             outputs) of blank and of every label position, gathered once so that the
//             recursions read them coalesced (small alphabets: the normalised rows themselves,
//             stored symbol-major)
//   lattice   alpha and beta recursions, both in one launch, a workgroup per utterance and direction
//             (cost only: alpha alone; alignment: the max recursion with recorded choices)
//   gradient  softmax minus the normalised per-symbol occupancy; zero fill of padding
//             (alignment: the backtrace instead)
//
// The recursions run on probabilities, each lane's values in fp64 with an int32 exponent of
// the lane's own (its "frame") that is renewed every kChunk steps: no transcendentals and a
// third of the instructions of the log-space form (run_chain_linear, run_chain_linear2).
// alpha and beta span thousands of binary orders of magnitude over a 15 s utterance, and the
// states that carry the mass lie a thousand orders below the largest of their frame, so the
// exponent has to be per lane; fp64 then leaves room for the kChunk steps between renewals.
// Utterances with an emission below 2^kLinearMinLog2 (found by the softmax launch), launches
// of the barrier kernel and the maximum recursion use the log-space form instead
// (run_chain_log): base-2 logarithms in fp64 (v_exp_f32 / v_log_f32 are base 2, so no scaling
// multiplies; only the bounded differences that enter them are narrowed to fp32), log(0) a
// large finite negative number, which keeps every operation NaN-free.
// Either way the lattice is stored as value words and exponent rows, see "lattice storage".

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
// log2 of a softmax output from the logit, the row's largest logit and log2 of the row's sum of
// 2^((x - max) log2 e).  The difference comes first: formed as x log2 e - (max log2 e + log2 sum) the
// result would carry the rounding of the offset, 6e-8 of its size, and a row of logits of size 100 whose
// winner has probability 1 - 1e-6 would give that winner an emission wrong by 1e-5, frame after frame.
__device__ __forceinline__ float log2_softmax(float x, float row_max, float log2_sum)
{
    return fmaf(x - row_max, kLog2e, -log2_sum);
}

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

// 16-byte vectors of activations: 4 floats or 8 bf16.
template <typename T> struct Vec;
template <> struct Vec<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void load(const float* p, float (&v)[4])
    {
        const float4 r = *reinterpret_cast<const float4*>(p);
        v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
    }
    static __device__ __forceinline__ void store(float* p, const float (&v)[4])
    {
        // Streaming store: the wide gradient is written once and not read again by this call
        // except in the few label columns (measured 7 % faster than a plain store on the
        // 6000-symbol workload, and the later fix-up of the label columns 20 % faster).
        typedef float v4f __attribute__((ext_vector_type(4)));
        const v4f t = {v[0], v[1], v[2], v[3]};
        __builtin_nontemporal_store(t, reinterpret_cast<v4f*>(p));
    }
};
template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[8])
    {
        const uint4 r = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8])
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = static_cast<uint32_t>(to_bf16_bits(v[2 * i])) |
                   (static_cast<uint32_t>(to_bf16_bits(v[2 * i + 1])) << 16);
        typedef uint32_t v4u __attribute__((ext_vector_type(4)));
        const v4u t = {w[0], w[1], w[2], w[3]};
        __builtin_nontemporal_store(t, reinterpret_cast<v4u*>(p));
    }
};

// ---- workgroup reductions (256 threads = 4 wavefronts), fixed order => repeatable -------

// Lane permutations inside a row of 16 lanes, as DPP operands of the add / max itself (no trip
// through the LDS crossbar): neighbours, pairs, then the mirrored half-row and the mirrored row.
template <int kCtrl>
__device__ __forceinline__ float dpp_permute(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), kCtrl, 0xf, 0xf, true));
}
// Every lane receives the sum (maximum) over its row of 16 lanes.  All 16 lanes must be active.
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_permute<0xB1>(v);      // quad_perm [1,0,3,2]
    v += dpp_permute<0x4E>(v);      // quad_perm [2,3,0,1]
    v += dpp_permute<0x141>(v);     // row_half_mirror
    v += dpp_permute<0x140>(v);     // row_mirror
    return v;
}
__device__ __forceinline__ float row16_max(float v)
{
    v = fmaxf(v, dpp_permute<0xB1>(v));
    v = fmaxf(v, dpp_permute<0x4E>(v));
    v = fmaxf(v, dpp_permute<0x141>(v));
    v = fmaxf(v, dpp_permute<0x140>(v));
    return v;
}
// The same over groups of 4 neighbouring lanes.
__device__ __forceinline__ float quad_sum(float v)
{
    v += dpp_permute<0xB1>(v);
    v += dpp_permute<0x4E>(v);
    return v;
}
__device__ __forceinline__ float quad_max(float v)
{
    v = fmaxf(v, dpp_permute<0xB1>(v));
    v = fmaxf(v, dpp_permute<0x4E>(v));
    return v;
}
__device__ __forceinline__ int quad_sum(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, true);
    return v;
}
// Whole wavefront (all 64 lanes active); the four row results are combined in a fixed order.
__device__ __forceinline__ float wave_sum(float v)
{
    const int r = __float_as_int(row16_sum(v));
    return (__int_as_float(__builtin_amdgcn_readlane(r, 0)) + __int_as_float(__builtin_amdgcn_readlane(r, 16))) +
           (__int_as_float(__builtin_amdgcn_readlane(r, 32)) + __int_as_float(__builtin_amdgcn_readlane(r, 48)));
}
__device__ __forceinline__ float wave_max(float v)
{
    const int r = __float_as_int(row16_max(v));
    return fmaxf(fmaxf(__int_as_float(__builtin_amdgcn_readlane(r, 0)), __int_as_float(__builtin_amdgcn_readlane(r, 16))),
                 fmaxf(__int_as_float(__builtin_amdgcn_readlane(r, 32)), __int_as_float(__builtin_amdgcn_readlane(r, 48))));
}

// Inclusive running sum over the 64 lanes of a wavefront (all active): lane i receives
// v_0 + ... + v_i, added up in a fixed order.  Four shifted additions within each row of 16
// lanes, then the last lane of a row is added to the rows above it (row_bcast).
template <int kCtrl, int kRowMask>
__device__ __forceinline__ float dpp_or_zero(float v)     // lanes without a source lane, or outside the rows, get 0
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), kCtrl, kRowMask, 0xf, false));
}
__device__ __forceinline__ float wave_running_sum(float v)
{
    v += dpp_or_zero<0x111, 0xf>(v);      // row_shr:1
    v += dpp_or_zero<0x112, 0xf>(v);      // row_shr:2
    v += dpp_or_zero<0x114, 0xf>(v);      // row_shr:4
    v += dpp_or_zero<0x118, 0xf>(v);      // row_shr:8
    v += dpp_or_zero<0x142, 0xa>(v);      // row_bcast:15 into rows 1 and 3
    v += dpp_or_zero<0x143, 0xc>(v);      // row_bcast:31 into rows 2 and 3
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

// ---- upload --------------------------------------------------------------------------------
// First launch of a call.  The per-call metadata (utterance records, run order, labels) was
// written by the host into pinned host memory; this kernel copies it word by word into the
// workspace, every read in flight at once, so that no stream-ordered copy-engine transfer
// (about 18 us of latency per call) sits between two calls.
// Where the image also holds the labels as bytes (alphabets of at most 256 symbols), the label words
// [labels_first, labels_end) are made from those: a quarter of the bytes over PCIe for what is most
// of the image (512 utterances of 29 symbols: 171 KB -> 67 KB, 8.7 -> 5.8 us).
__global__ __launch_bounds__(kRowThreads)
void ctc_upload_kernel(const int* __restrict__ host_image, int* __restrict__ ws, int words,
                       int labels_first, int labels_end, const unsigned char* __restrict__ labels8)
{
    const int i = blockIdx.x * kRowThreads + threadIdx.x;
    if (i >= words) return;
    if (labels8 && i >= labels_first && i < labels_end)
        ws[i] = labels8[i - labels_first];
    else
        ws[i] = host_image[i];
}

// ---- device-side planning -------------------------------------------------------------------
// The device-metadata entry point has no host image: lengths and labels are device arrays that
// the host never sees, so this kernel (one workgroup) does what the host launcher does
// otherwise.  Per utterance: range checks, the count of adjacent repeats (an alignment exists
// iff T_b >= L + repeats), the wavefront plan, and the offsets of its blocks, which are laid
// out with the strides of the largest utterance the caller allows (labels [B][max_label],
// emissions b * T * max_label, lattice b * T * lattice_pitch(max_label), frames b * T).  Then the run
// order: heaviest chains first (rank by T_b x wavefronts, ties by index), -1 for the rest.
constexpr int kPlanThreads = 1024;

__global__ __launch_bounds__(kPlanThreads)
void ctc_plan_kernel(const int* __restrict__ labels, const int* __restrict__ label_lengths,
                     const int* __restrict__ input_lengths, Utt* __restrict__ meta,
                     int* __restrict__ order, int* __restrict__ status,
                     int Tt, int B, int A, int blank, int max_label, int poll_budget, bool crowded,
                     bool log_domain, int dirs)
{
    __shared__ long long weight[kMaxDeviceMetaB];     // T_b x wavefronts; -1: does not run
    __shared__ int repeats[kMaxDeviceMetaB];          // adjacent equal symbols; kBadLabel added for a bad symbol
    __shared__ int s_bad, s_running;
    constexpr int kBadLabel = 1 << 20;
    const int tid = threadIdx.x;
    if (tid == 0) {
        s_bad = 0;
        s_running = 0;
    }
    int* const s_len = reinterpret_cast<int*>(weight);       // label lengths, until the weights are written
    for (int i = tid; i < B; i += kPlanThreads) {
        order[2 * i] = -1;
        order[2 * i + 1] = -1;
        repeats[i] = 0;
        s_len[i] = label_lengths[i];
    }
    __syncthreads();
    // Every entry of the padded label matrix on its own, eight reads per thread in flight.
    const int cells = B * max_label;
    for (int i0 = tid; i0 < cells; i0 += 8 * kPlanThreads) {
        int c[8], before[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u * kPlanThreads;
            c[u] = (i < cells) ? labels[i] : 0;
            before[u] = (i < cells && i > 0) ? labels[i - 1] : -1;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u * kPlanThreads;
            if (i >= cells) continue;
            const int b = i / max_label, j = i - b * max_label;
            const int L = s_len[b];
            if (j < L && L <= max_label) {
                int add = (c[u] < 0 || c[u] >= A || c[u] == blank) ? kBadLabel : 0;
                if (j > 0 && c[u] == before[u]) ++add;
                if (add) atomicAdd(&repeats[b], add);
            }
        }
    }
    __syncthreads();
    for (int b = tid; b < B; b += kPlanThreads) {
        const int L = label_lengths[b], Tb = input_lengths[b];
        const int rep = repeats[b];
        const bool bad = L < 0 || L > max_label || Tb < 0 || Tb > Tt || rep >= kBadLabel;
        const bool runs = !bad && Tb > 0 && Tb >= L + rep;
        const WavePlan wp = plan_waves(bad ? 0 : L, crowded);
        Utt m;
        m.Tb = bad ? 0 : Tb;
        m.L = bad ? 0 : L;
        m.lab_off = b * max_label;
        m.flags = (runs ? kUttRuns : 0) | (bad ? kUttInvalid : 0) |
                  ((log_domain || Tb > kLinearMaxFrames || tight_fit(Tb, L, rep)) ? kUttLogDomain : 0) |
                  (!bad && two_pairs_per_lane(L, crowded, emission_layout(A) == kEmitSymbolMajor) ? kUttTwoPairs : 0);
        m.f_off = b * Tt;
        m.waves = wp.waves;
        m.halo = wp.halo;
        const WavePlan wp2 = plan_waves2(bad ? 0 : L, crowded);
        m.waves2 = wp2.waves;
        m.halo2 = wp2.halo;
        m.poll_budget = poll_budget;
        m.e_direct = emission_layout(A);
        m.e_pitch = m.e_direct == kEmitSymbolMajor ? Tt : m.L;
        m.e_off = static_cast<int64_t>(b) * Tt * (m.e_direct ? A : max_label);
        m.ab_off = static_cast<int64_t>(b) * Tt * lattice_pitch(max_label);
        meta[b] = m;
        weight[b] = runs ? static_cast<long long>(Tb) * ((m.flags & kUttTwoPairs) ? wp2.waves : wp.waves) : -1;
        if (bad) s_bad = 1;
        if (runs) atomicAdd(&s_running, 1);
    }
    __syncthreads();
    if (tid == 0) *status = s_bad ? CTC_STATUS_INVALID_VALUE : CTC_STATUS_SUCCESS;
    for (int i = tid; i < B; i += kPlanThreads) {
        const long long wi = weight[i];
        if (wi < 0) continue;
        int rank = 0;
        for (int j = 0; j < B; ++j) {
            const long long wj = weight[j];
            rank += (wj > wi) || (wj == wi && j < i);
        }
        // Heaviest first, in blocks of kChainBlock utterances: a block's forward chains, then its
        // backward chains (order_chains; the device planner does not balance the SIMDs' loads
        // beyond that).
        const int first = rank - rank % kChainBlock, in_block = min(kChainBlock, s_running - first);
        for (int d = 0; d < dirs; ++d) order[first * dirs + d * in_block + rank % kChainBlock] = 2 * i + d;
    }
}

// ---- setup role ----------------------------------------------------------------------------
// Runs in one extra grid column of the softmax launch, one workgroup per utterance, beside
// the row work.  It groups the label positions by symbol, once per utterance, for every frame
// of the gradient to reuse -- the purpose of the appendix's one-off key-value sort of the
// label.  Word of label position j:
//   bits  0..9   its slot in the order (symbol ascending, then position ascending): the
//                positions of one symbol occupy consecutive slots
//   bits 12..21  how often its symbol occurs in the label
//   bit  31      set if j is the first occurrence of its symbol (its slot then starts the run)
// The gradient kernels write each state's mass share to its slot and let the first occurrence
// add up the run in slot order, so a symbol's occupancy has one writer and a fixed order of
// summation.  Also here: costs of utterances without a lattice, the per-utterance error
// flags, the two constants of the emission array.
constexpr int kLinkSlotMask = 0x3FF, kLinkCountShift = 12;
static_assert(CTC_MAX_LABEL_LENGTH <= kLinkSlotMask, "slot and count fields hold 10 bits");

// (The constants that lanes without a label state read as their emission, kZeroEmission and
// kLogZeroEmission, are laid out in the launcher's header, with the chains' fetch schedule.)

struct SetupArgs {
    int* links;
    float* costs;
    int* chain_err;
    int* done;            // per utterance: wavefronts of its chains that have ended (overlapped launches)
    int* where;           // per chain: the die it runs on
    int* leftover;        // per utterance: rows left to the gradient launch
    float* log0;          // kEmissionConstants floats that lattice lanes without a label state read as their
                          // emission: probability 0 (linear-domain chains) and log 0 (log-domain chains)
    double* emit_blank64; // the blank's probability per frame as fp64 (Layout::emit_blank64)
    int* host_flag;       // pinned host word: receives flag_value once the upload has been consumed
    int flag_value;
    bool plain_logs;      // emissions are stored as log2 probabilities throughout (most probable alignment)
    int parts;            // workgroups per utterance that share the setup role (grid columns beyond the rows)
};

// The grouping compares every pair of label positions; it is spread over `parts` workgroups per
// utterance (64 positions each at a time) and four lanes per position, each lane walking a quarter
// of the label, so that a label of 500 symbols costs 125 steps per lane instead of 1000.
constexpr int kSetupLabelSlots = CTC_MAX_LABEL_LENGTH + 5;     // the label and a quarter's padding

// `labels8`: the label strings as bytes (narrow alphabets, read out of the pinned host image: a
// quarter of the traffic), to be written out as ints to `labels_out` by the utterance's first part;
// nullptr: `labels` holds them as ints.
__device__ __forceinline__ void setup_words(const Utt m, const int b, const SetupArgs sa);
// (`with_words`: the utterance's first part also writes its setup_words)
__device__ __forceinline__ void setup_role(const Utt m, const int b, const int* __restrict__ labels,
                                           const SetupArgs sa, int* s_lab, const int part, const int parts,
                                           const unsigned char* __restrict__ labels8 = nullptr,
                                           int* __restrict__ labels_out = nullptr, const bool with_words = true)
{
    const int tid = threadIdx.x;
    const int* lab = labels + m.lab_off;
    const int quarter_length = (m.L + 3) / 4;
    // padding: a symbol that is neither smaller than nor equal to any real one
    for (int j = tid; j < 4 * quarter_length; j += kRowThreads) {
        const int c = (j >= m.L) ? 0x7FFFFFFF : (labels8 ? static_cast<int>(labels8[m.lab_off + j]) : lab[j]);
        s_lab[j] = c;
        if (labels_out && part == 0 && j < m.L) labels_out[m.lab_off + j] = c;
    }
    __syncthreads();
    const int quarter = tid & 3;
    const int* const mine = s_lab + quarter * quarter_length;
    const int first_i = quarter * quarter_length;
    for (int j = part * 64 + (tid >> 2); j < m.L; j += parts * 64) {
        const int c = s_lab[j];
        // Independent iterations keep the LDS reads in flight.
        int below = 0, before = 0, count = 0;
        for (int i = 0; i < quarter_length; ++i) {
            const int ci = mine[i];
            below += ci < c;
            count += ci == c;
            before += (ci == c) & (first_i + i < j);
        }
        below = quad_sum(below);
        count = quad_sum(count);
        before = quad_sum(before);
        if (quarter == 0)
            sa.links[m.lab_off + j] = (below + before) | (count << kLinkCountShift) |
                                      (before == 0 ? static_cast<int>(0x80000000u) : 0);
    }
    if (part == 0 && with_words) setup_words(m, b, sa);
}

// The per-utterance words that every call starts from, the constants of the emission array, and the costs
// of utterances without a lattice.  By one workgroup per utterance.
__device__ __forceinline__ void setup_words(const Utt m, const int b, const SetupArgs sa)
{
    if (threadIdx.x == 0) {
        sa.chain_err[b] = 0;
        sa.done[b * kDoneStride] = 0;
        sa.where[2 * b] = 0;
        sa.where[2 * b + 1] = 0;
        sa.leftover[b] = (m.flags & kUttGradientLater) ? 1 : 0;
        if (b == 0) {
            for (int i = 0; i < kEmissionConstants; ++i) sa.log0[i] = (i < kEmissionConstantRun) ? 0.0f : static_cast<float>(kNeg);
            // This launch follows the upload kernel on the stream, so the host may now reuse
            // the pinned image.
            if (sa.host_flag)
                __hip_atomic_store(sa.host_flag, sa.flag_value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        // No frames: the empty product (cost 0) for an empty label.  Otherwise no alignment.
        if (m.flags & kUttInvalid) sa.costs[b] = __uint_as_float(0x7FC00000u);
        else if (!(m.flags & kUttRuns)) sa.costs[b] = (m.Tb == 0 && m.L == 0) ? 0.0f : __builtin_inff();
    }
}

// ---- emission coding -------------------------------------------------------------------------
// The recursions run on probabilities (linear domain, see run_chain_linear) unless some
// emission of the utterance is too small for that; an emission is therefore stored as the
// probability y = 2^lp itself, or, where lp < kLinearMinLog2, as lp (a negative float, which
// no probability is).  A lane that stores such a value raises the utterance's kUttLogDomain
// flag, and its chains then take log2 of the stored probabilities instead.
// (The most probable alignment has no sums to speed up: its launches store plain logarithms.)
__device__ __forceinline__ float encode_emission(float lp, bool& small, bool plain_logs)
{
    if (plain_logs) return lp;
    if (lp >= kLinearMinLog2) return fast_exp2(lp);
    small = true;
    return lp;
}
// log2 of a coded emission in two floats whose sum it is: the binary exponent of a stored probability
// and the logarithm of its mantissa.  (As one float the logarithm of 2^-40 would be good to 4e-6 only,
// frame after frame; a chain of 400 steps then misses the gradient's bound.)
struct Log2Parts { float whole, part; };
__device__ __forceinline__ Log2Parts emission_log2_parts(float v)
{
    if (v > 0.0f)
        return {static_cast<float>(__builtin_amdgcn_frexp_expf(v)), fast_log2(__builtin_amdgcn_frexp_mantf(v))};
    return {v, 0.0f};
}
__device__ __forceinline__ double emission_log2(float v)
{
    const Log2Parts p = emission_log2_parts(v);
    return static_cast<double>(p.whole) + static_cast<double>(p.part);
}
__device__ __forceinline__ float emission_probability(float v) { return fmaxf(v, 0.0f); }
__device__ __forceinline__ void raise_log_domain(Utt* meta, int b, bool small)
{
    if (small) atomicOr(&meta[b].flags, kUttLogDomain);
}

// ---- softmax statistics + emission gather --------------------------------------------------
// Wide alphabets (A > 2048): one workgroup per row (t, b) of the tensor; grid (T + 1, B) for the
// scalar kernel, (B, T + 1) for the vector kernel; the extra column (row) does the setup role.
// The gradient of a wide alphabet is the softmax itself except in the few columns whose symbol
// occurs in the label, so these kernels also write the dense part of the gradient while they
// hold the row: y for valid rows, zeros for padding rows and for utterances without an
// alignment (skipped when no gradient is asked for: grads == nullptr).  The activations are then never read a second time; the label columns are
// corrected after the recursions by the sparse variant of the gradient kernel.
template <typename T>
__global__ __launch_bounds__(kRowThreads)
void ctc_softmax_kernel(const T* __restrict__ x, T* __restrict__ grads,
                        Utt* __restrict__ meta,
                        const int* __restrict__ labels, float* __restrict__ lse,
                        float* __restrict__ emit_blank, float* __restrict__ emit_label,
                        const SetupArgs sa, int Tt, int B, int A, int blank)
{
    __shared__ float red[8];
    __shared__ int s_lab[kSetupLabelSlots];
    const int t = blockIdx.x, b = blockIdx.y;
    const Utt m = meta[b];
    if (t == Tt) { setup_role(m, b, labels, sa, s_lab, 0, 1); return; }
    const size_t row_off = (static_cast<size_t>(t) * B + b) * A;
    T* grow = grads + row_off;
    const bool runs = (m.flags & kUttRuns) != 0;
    if (t >= m.Tb || !runs) {
        if (grads)
            for (int k = threadIdx.x; k < A; k += kRowThreads) store_elem(grow, k, 0.0f);
        return;
    }
    const T* row = x + row_off;

    float mx = -__builtin_inff();
    for (int k = threadIdx.x; k < A; k += kRowThreads) mx = fmaxf(mx, load_elem(row, k));
    mx = block_max(mx, red);
    float s = 0.0f;
    for (int k = threadIdx.x; k < A; k += kRowThreads)
        s += fast_exp2((load_elem(row, k) - mx) * kLog2e);
    s = block_sum(s, red + 4);
    // log2 y_k = (x_k - max) log2 e - log2 sum: the difference first, so that the error is relative to
    // log2 y_k itself and not to the row's offset (see log2_softmax)
    const float ls = fast_log2(s);
    const float l2 = fmaf(mx, kLog2e, ls);
    if (threadIdx.x == 0) lse[static_cast<size_t>(b) * Tt + t] = l2;

    if (grads)
        for (int k = threadIdx.x; k < A; k += kRowThreads)
            store_elem(grow, k, fast_exp2(log2_softmax(load_elem(row, k), mx, ls)));
    bool small = false;
    if (threadIdx.x == 0)
    {
        const float e = encode_emission(log2_softmax(load_elem(row, blank), mx, ls), small, sa.plain_logs);
        emit_blank[kBlankSlack + m.f_off + t] = e;
        sa.emit_blank64[kBlankSlack + m.f_off + t] = static_cast<double>(emission_probability(e));
    }
    float* erow = emit_label + kLabelSlack + m.e_off + static_cast<size_t>(t) * m.L;
    const int* lab = labels + m.lab_off;
    for (int j = threadIdx.x; j < m.L; j += kRowThreads)
        erow[j] = encode_emission(log2_softmax(load_elem(row, lab[j]), mx, ls), small, sa.plain_logs);
    raise_log_domain(meta, b, small);
}

// Wide alphabets, 16-byte aligned rows of at most 8192 symbols: the row is read once with
// 16-byte loads and stays in registers between the maximum and the sum.
constexpr int kWideMaxA = 8192;

template <typename T>
__global__ __launch_bounds__(kRowThreads)
void ctc_softmax_wide_kernel(const T* __restrict__ x, T* __restrict__ grads,
                             Utt* __restrict__ meta,
                             const int* __restrict__ labels, float* __restrict__ lse,
                             float* __restrict__ emit_blank, float* __restrict__ emit_label,
                             const SetupArgs sa, int Tt, int B, int A, int blank)
{
    constexpr int N = Vec<T>::N;
    constexpr int kVecs = kWideMaxA / (N * kRowThreads);      // vectors per thread
    __shared__ float red[8];
    __shared__ int s_lab[kSetupLabelSlots];
    // Utterance fastest: consecutive workgroups take consecutive rows of the tensor.
    const int t = blockIdx.y, b = blockIdx.x, tid = threadIdx.x;
    const Utt m = meta[b];
    if (t == Tt) { setup_role(m, b, labels, sa, s_lab, 0, 1); return; }
    const size_t row_off = (static_cast<size_t>(t) * B + b) * A;
    T* grow = grads + row_off;
    const int nvec = A / N;
    const bool runs = (m.flags & kUttRuns) != 0;
    if (t >= m.Tb || !runs) {
        const float zero[N] = {};
        if (grads)
            for (int i = tid; i < nvec; i += kRowThreads) Vec<T>::store(grow + static_cast<size_t>(i) * N, zero);
        return;
    }
    const T* row = x + row_off;

    float v[kVecs][N];
    float mx = -__builtin_inff();
#pragma unroll
    for (int i = 0; i < kVecs; ++i) {
        const int idx = tid + i * kRowThreads;
        if (idx < nvec) {
            Vec<T>::load(row + static_cast<size_t>(idx) * N, v[i]);
#pragma unroll
            for (int e = 0; e < N; ++e) mx = fmaxf(mx, v[i][e]);
        }
    }
    mx = block_max(mx, red);
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < kVecs; ++i) {
        if (tid + i * kRowThreads < nvec) {
#pragma unroll
            for (int e = 0; e < N; ++e) sum += fast_exp2((v[i][e] - mx) * kLog2e);
        }
    }
    sum = block_sum(sum, red + 4);
    const float ls = fast_log2(sum);
    const float l2 = fmaf(mx, kLog2e, ls);
    if (tid == 0) lse[static_cast<size_t>(b) * Tt + t] = l2;

#pragma unroll
    for (int i = 0; i < kVecs; ++i) {
        const int idx = tid + i * kRowThreads;
        if (grads && idx < nvec) {
            float y[N];
#pragma unroll
            for (int e = 0; e < N; ++e) y[e] = fast_exp2(log2_softmax(v[i][e], mx, ls));
            Vec<T>::store(grow + static_cast<size_t>(idx) * N, y);
        }
    }
    bool small = false;
    if (tid == 0)
    {
        const float e = encode_emission(log2_softmax(load_elem(row, blank), mx, ls), small, sa.plain_logs);
        emit_blank[kBlankSlack + m.f_off + t] = e;
        sa.emit_blank64[kBlankSlack + m.f_off + t] = static_cast<double>(emission_probability(e));
    }
    float* erow = emit_label + kLabelSlack + m.e_off + static_cast<size_t>(t) * m.L;
    const int* lab = labels + m.lab_off;
    for (int j = tid; j < m.L; j += kRowThreads)
        erow[j] = encode_emission(log2_softmax(load_elem(row, lab[j]), mx, ls), small, sa.plain_logs);
    raise_log_domain(meta, b, small);
}

// Narrow alphabets: a workgroup takes kRows consecutive frames of one utterance, 256 / kRows
// threads per row.  The normalised rows (as coded emissions) are kept in LDS
// (kRows * A floats, dynamic), from where the emissions of all label positions are gathered
// with the label symbols held in registers.  grid (ceil(T / kRows) + 1, B), the extra column
// does the setup role.
template <typename T, int kRows>
__global__ __launch_bounds__(kRowThreads)
void ctc_softmax_rows_kernel(const T* __restrict__ x, Utt* __restrict__ meta,
                             const int* __restrict__ labels, float* __restrict__ lse,
                             float* __restrict__ emit_blank, float* __restrict__ emit_label,
                             const SetupArgs sa, int Tt, int B, int A, int blank)
{
    constexpr int kPerRow = kRowThreads / kRows;          // threads per row: a quad, a 16-lane row or a wavefront
    static_assert(kPerRow == 4 || kPerRow == 16 || kPerRow == 64, "row reductions exist for 4, 16 and 64 lanes");
    extern __shared__ float lp[];                          // [kRows][A]
    __shared__ int s_lab[kSetupLabelSlots];
    const int b = blockIdx.y, tid = threadIdx.x;
    const Utt m = meta[b];
    if (blockIdx.x >= gridDim.x - sa.parts) {
        setup_role(m, b, labels, sa, s_lab, static_cast<int>(blockIdx.x - (gridDim.x - sa.parts)), sa.parts);
        return;
    }
    const int t0 = blockIdx.x * kRows;
    if (t0 >= m.Tb) return;
    const int r = tid / kPerRow, q = tid % kPerRow, t = t0 + r;
    float* lrow = lp + r * A;
    // Requested before the row work so that its latency overlaps the row's.
    const int* lab = labels + m.lab_off;
    const int c_first = (!m.e_direct && tid < m.L) ? lab[tid] : 0;
    if (t < m.Tb) {
        const T* row = x + (static_cast<size_t>(t) * B + b) * A;
        float mx = -__builtin_inff();
        // eight reads in flight per thread: a row costs a few memory latencies, not A / kPerRow
        for (int k0 = q; k0 < A; k0 += 8 * kPerRow) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int k = k0 + u * kPerRow;
                v[u] = (k < A) ? load_elem(row, k) : -__builtin_inff();
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int k = k0 + u * kPerRow;
                if (k < A) lrow[k] = v[u];
                mx = fmaxf(mx, v[u]);
            }
        }
        mx = (kPerRow == 4) ? quad_max(mx) : (kPerRow == 16) ? row16_max(mx) : wave_max(mx);
        float sum = 0.0f;
        for (int k = q; k < A; k += kPerRow) sum += fast_exp2((lrow[k] - mx) * kLog2e);
        sum = (kPerRow == 4) ? quad_sum(sum) : (kPerRow == 16) ? row16_sum(sum) : wave_sum(sum);
        const float ls = fast_log2(sum);
        const float l2 = fmaf(mx, kLog2e, ls);
        // (coded as emissions; `unused` because what counts is which of them get stored below)
        bool unused = false;
        for (int k = q; k < A; k += kPerRow) lrow[k] = encode_emission(log2_softmax(lrow[k], mx, ls), unused, sa.plain_logs);
        if (q == 0) lse[static_cast<size_t>(b) * Tt + t] = l2;
    }
    if (!(m.flags & kUttRuns)) return;
    __syncthreads();
    const int rows = min(kRows, m.Tb - t0);
    bool small = false;
    if (tid < rows) {
        const float e = lp[tid * A + blank];
        emit_blank[kBlankSlack + m.f_off + t0 + tid] = e;
        sa.emit_blank64[kBlankSlack + m.f_off + t0 + tid] = static_cast<double>(emission_probability(e));
        small = !sa.plain_logs && e < 0.0f;
    }
    if (m.e_direct == kEmitSymbolMajor) {
        // Small alphabet: the normalised rows themselves are the emission block, stored symbol-major
        // (a symbol's frames side by side, e_pitch floats per symbol: fetch_frames).  A wavefront
        // writes up to 64 frames of one symbol at a time.
        float* out = emit_label + kLabelSlack + m.e_off + t0;
        const int rr = tid & 63;
        if (rr < rows)
            for (int a = tid >> 6; a < A; a += kRowThreads / 64) {
                const float e = lp[rr * A + a];
                out[static_cast<size_t>(a) * m.e_pitch + rr] = e;
                small = small || (!sa.plain_logs && e < 0.0f);
            }
        raise_log_domain(meta, b, small);
        return;
    }
    float* ebase = emit_label + kLabelSlack + m.e_off + static_cast<size_t>(t0) * m.L;
    for (int j = tid; j < m.L; j += kRowThreads) {
        const int c = (j == tid) ? c_first : lab[j];
        for (int rr = 0; rr < rows; ++rr) {
            const float e = lp[rr * A + c];
            ebase[static_cast<size_t>(rr) * m.L + j] = e;
            small = small || (!sa.plain_logs && e < 0.0f);
        }
    }
    raise_log_domain(meta, b, small);
}

// The narrowest alphabets (at most kDirectMaxA symbols), host-resident metadata: the first launch of
// the call.  There is no upload launch before it: every workgroup reads its utterance's record out
// of the pinned host image itself (one PCIe round trip, which the upload launch cost as well, but
// no launch boundary after it), and the workgroups of the setup role, besides their own work, copy
// the image into the workspace for the launches that follow.  Nothing in this launch writes where
// another of its workgroups reads: instead of raising a flag in the utterance's record, a workgroup
// that meets an emission too small for the linear domain says so in a word of its own
// (row_flags: one per kFlagFrames frames of an utterance, written by every workgroup that has rows),
// which the chains gather when they start.
// A workgroup takes 64 frames of one utterance, four lanes per frame, so that it has several
// kilobytes under way; the normalised rows are the emission block, stored symbol-major.
// grid (ceil(T / 64) + parts, B); dynamic LDS 64 * A floats.
struct NarrowImage {
    const int* words;         // the pinned image: meta, order, labels, tasks as they lie in the workspace, then the labels as bytes
    int labels_first, labels_end;   // the label strings' place in it (4-byte words): not copied, the setup role writes them
    int count;                // words to copy (up to the byte labels)
    size_t labels8_offset;    // of the byte labels (bytes)
    int* labels_out;          // the workspace's label strings
};
// What the workgroups with rows need to know of an utterance travels with the kernel's arguments
// (hundreds of small reads out of host memory at once were measured to take longer than the upload
// launch they replace): its frames, with kRowsRun set if its chains run, and the frames of all
// utterances before it.  An utterance's emission block starts A times that many floats into the
// region and has a pitch of its frames.
constexpr int kRowsRun = 1 << 30, kRowsGradientLater = 1 << 29;     // (flags of the record that ride along)
struct NarrowRows {
    int frames[kNarrowMaxB];
    int frames_before[kNarrowMaxB];
    int label_length[kNarrowMaxB];       // and, for the setup role, the label's length and the symbols before it
    int labels_before[kNarrowMaxB];
};
// Either that (host-resident metadata) or the wavefront plans by label length (device-resident
// metadata: see NarrowDevice), in the same 2 KB of kernel arguments.
union NarrowArgs {
    NarrowRows rows;
    PlanTable plans;
};

// Device-resident metadata (ctc_loss_and_grad_device): there is no image and there are no records
// yet.  The workgroups with rows derive what they need from the lengths themselves (blocks are laid
// out by the caller's bounds: see ctc_plan_kernel); the first setup workgroup of an utterance builds
// its record, as ctc_plan_kernel does for wider alphabets in a launch of its own, and finds the
// utterance's place in the run order by counting the utterances that weigh more (all utterances
// take part, those without an alignment too: their chains' workgroups leave at once).
struct NarrowDevice {
    const int* labels;            // [B][max_label]; nullptr: the metadata is the host's (NarrowImage, NarrowRows)
    const int* label_lengths;
    const int* input_lengths;
    Utt* meta;                    // records to build
    int* order;
    int* status_words;            // [B] nonzero: the utterance's lengths or labels are invalid
    int max_label, poll_budget, dirs;
    bool crowded, log_domain;
    int* tasks;                   // the lattice launch's workers' task list, to be built here (nullptr: no workers)
    int share_percent;            // utterances whose chains end later than this share of the longest go to the gradient launch
    int n_cu;                     // compute units of the device (a multiple of kChainBlock, or 0: keep the plain order)
};

// Wavefronts of an utterance's chains (0: its lengths are out of range).
__device__ __forceinline__ int chain_waves(const PlanTable& plans, int L, int Tb, int Tt, int max_label, bool log_domain)
{
    if (L < 0 || L > max_label || Tb < 0 || Tb > Tt) return 0;
    const bool two = !log_domain && Tb <= kLinearMaxFrames && plans.two_pairs(L);
    return two ? plans.waves2(L) : plans.waves1(L);
}
// Weight of an utterance in the run order: its frames times the wavefronts of its chains.
__device__ __forceinline__ long long chain_weight(const PlanTable& plans, int L, int Tb, int Tt, int max_label,
                                                  bool log_domain)
{
    return static_cast<long long>(Tb) * chain_waves(plans, L, Tb, Tt, max_label, log_domain);
}
// When an utterance's chains end, in the unit the launcher orders by (prepare: chains that exchange
// between wavefronts take a little longer per frame); 0 for an utterance without frames or with bad lengths.
__device__ __forceinline__ int chain_end_estimate(const PlanTable& plans, int L, int Tb, int Tt, int max_label, bool log_domain)
{
    const int waves = chain_waves(plans, L, Tb, Tt, max_label, log_domain);
    return waves == 0 ? 0 : Tb * (waves > 1 ? 5 : 4);
}
__device__ __forceinline__ bool ends_late(int ends, int last_end, int share_percent)
{
    return static_cast<long long>(ends) * 100 > static_cast<long long>(last_end) * share_percent;
}

// The workers' task list (see gradient_worker and the launcher's prepare, whose list this reproduces from the
// device-resident lengths), by one workgroup.  An utterance's place in the run order is its rank by weight
// over all B utterances (build_record), its chains' die that rank mod kXcds (the order's blocks of kChainBlock
// keep both chains of an utterance on one die; in a last, partial block they may not be, and a worker that
// finds them elsewhere leaves the utterance to the gradient launch).  Whether an alignment exists is not
// looked at: the workers take that from the records.  B <= kMaxTaskEntries / 2.
__device__ __forceinline__ void build_task_table(const NarrowDevice& dv, const PlanTable& plans, int Tt, int B)
{
    constexpr int kMax = kMaxTaskEntries / 2;
    static_assert(kRowThreads == 2 * kMax, "two threads per utterance");
    __shared__ long long s_weight[kMax];
    __shared__ int s_frames[kMax], s_ends[kMax], s_rank[kMax], s_wait[kMax], s_pad[kMax], s_at[kMax], s_sum[kMax];
    __shared__ int s_last_end, s_entries[kXcds][2], s_tasks[kXcds][2];      // per die: [padding rows, waiting rows]
    __shared__ int s_entries_before[kXcds + 1], s_tasks_before[kXcds + 1];
    const int tid = threadIdx.x, blocks = (Tt + kTaskRows - 1) / kTaskRows;
    // Four threads per utterance j (two beyond 64 utterances), each comparing it with a quarter (half) of the
    // others in one unrolled pass, so that its LDS reads travel together; entries beyond B are neutral.
    const int span = B <= kMax / 2 ? kMax / 2 : kMax, share = span / (kRowThreads / span);
    const int j = tid & (span - 1), k_first = (tid / span) * share, k_end = k_first + share;
    if (tid == 0) s_last_end = 0;
    if (tid < kXcds * 2) {
        s_entries[tid >> 1][tid & 1] = 0;
        s_tasks[tid >> 1][tid & 1] = 0;
    }
    if (tid < B) {
        const int L = dv.label_lengths[tid], Tb = dv.input_lengths[tid];
        s_weight[tid] = chain_weight(plans, L, Tb, Tt, dv.max_label, dv.log_domain);
        s_ends[tid] = chain_end_estimate(plans, L, Tb, Tt, dv.max_label, dv.log_domain);
        s_frames[tid] = Tb;
        s_rank[tid] = 0;
        s_at[tid] = 0;
        s_sum[tid] = 0;
    } else if (tid < kMax) {
        s_weight[tid] = -1;                             // (lighter than any utterance)
        s_ends[tid] = 0;
        s_rank[tid] = 0;
        s_wait[tid] = 0;
    }
    __syncthreads();
    if (tid < B && s_ends[tid] > 0) atomicMax(&s_last_end, s_ends[tid]);
    if (j < B) {
        const long long mine = s_weight[j];
        int before = 0;
#pragma unroll 16
        for (int k = k_first; k < k_end; ++k) before += (s_weight[k] > mine || (s_weight[k] == mine && k < j)) ? 1 : 0;
        if (before) atomicAdd(&s_rank[j], before);
    }
    __syncthreads();
    if (tid < B) {
        const int data = s_ends[tid] > 0 ? (s_frames[tid] + kTaskRows - 1) / kTaskRows : 0;
        s_pad[tid] = blocks - data;
        s_wait[tid] = ends_late(s_ends[tid], s_last_end, dv.share_percent) ? 0 : data;
        if (s_pad[tid] > 0) {
            atomicAdd(&s_entries[tid % kXcds][0], 1);
            atomicAdd(&s_tasks[tid % kXcds][0], s_pad[tid]);
        }
        if (s_wait[tid] > 0) {
            atomicAdd(&s_entries[s_rank[tid] % kXcds][1], 1);
            atomicAdd(&s_tasks[s_rank[tid] % kXcds][1], s_wait[tid]);
        }
    }
    __syncthreads();
    // a waiting entry's place in its die's section: the die's utterances that end earlier (ties: in the run order)
    if (j < B && s_wait[j] > 0) {
        const int die = s_rank[j] % kXcds, ends = s_ends[j], rank = s_rank[j];
        int at = 0, sum = 0;
#pragma unroll 16
        for (int k = k_first; k < k_end; ++k) {
            const int wait_k = s_wait[k], rank_k = s_rank[k], ends_k = s_ends[k];
            const bool earlier = wait_k > 0 && rank_k % kXcds == die && (ends_k < ends || (ends_k == ends && rank_k < rank));
            at += earlier ? 1 : 0;
            sum += earlier ? wait_k : 0;
        }
        if (at) {
            atomicAdd(&s_at[j], at);
            atomicAdd(&s_sum[j], sum);
        }
    }
    if (tid <= kXcds) {
        int entries = 0, tasks = 0;
        for (int d = 0; d < tid; ++d) {
            entries += s_entries[d][0] + s_entries[d][1];
            tasks += s_tasks[d][0] + s_tasks[d][1];
        }
        s_entries_before[tid] = entries;
        s_tasks_before[tid] = tasks;
    }
    __syncthreads();
    int* const task_die = dv.tasks;                     // [kXcds + 1]
    int* const task_prefix = task_die + kXcds + 1;      // [2B + 1]
    int* const task_info = task_prefix + 2 * B + 1;     // [2B]
    int* const task_first = task_info + 2 * B;          // [2B]
    if (tid < B) {
        if (s_pad[tid] > 0) {
            // the die's padding rows come first, by utterance number
            const int die = tid % kXcds;
            int at = 0, sum = 0;
            for (int k = die; k < tid; k += kXcds)
                if (s_pad[k] > 0) {
                    ++at;
                    sum += s_pad[k];
                }
            const int e = s_entries_before[die] + at;
            task_prefix[e] = s_tasks_before[die] + sum;
            task_info[e] = tid | (kTaskRowsLog2 << kTaskRowsShift);
            task_first[e] = blocks - s_pad[tid];
        }
        if (s_wait[tid] > 0) {
            // then its utterances as their chains end
            const int die = s_rank[tid] % kXcds;
            const int e = s_entries_before[die] + s_entries[die][0] + s_at[tid];
            task_prefix[e] = s_tasks_before[die] + s_tasks[die][0] + s_sum[tid];
            task_info[e] = tid | kTaskWaits | (kTaskRowsLog2 << kTaskRowsShift);
            task_first[e] = 0;
        }
    }
    if (tid <= kXcds) task_die[tid] = s_entries_before[tid];
    if (tid == 0) task_prefix[s_entries_before[kXcds]] = s_tasks_before[kXcds];
}

// By the whole workgroup; `s_lab` holds scratch ints.  Returns the record (the same in every thread).
__device__ __forceinline__ Utt build_record(const NarrowDevice& dv, const PlanTable& plans, int b, int Tt, int B, int A,
                                            int blank)
{
    __shared__ int s_repeats, s_bad, s_rank, s_last_end;
    const int tid = threadIdx.x;
    const int L_in = dv.label_lengths[b], Tb_in = dv.input_lengths[b];
    const bool bad_length = L_in < 0 || L_in > dv.max_label || Tb_in < 0 || Tb_in > Tt;
    const int L = bad_length ? 0 : L_in;
    if (tid == 0) {
        s_repeats = 0;
        s_bad = 0;
        s_rank = 0;
        s_last_end = 0;
    }
    __syncthreads();
    const int* lab = dv.labels + static_cast<size_t>(b) * dv.max_label;
    int repeats = 0, bad = 0;
    for (int j = tid; j < L; j += kRowThreads) {
        const int c = lab[j];
        bad |= (c < 0 || c >= A || c == blank) ? 1 : 0;
        repeats += (j > 0 && c == lab[j - 1]) ? 1 : 0;
    }
    if (repeats) atomicAdd(&s_repeats, repeats);
    if (bad) s_bad = 1;
    // the utterances that come before this one in the run order: heavier, or as heavy and earlier
    const long long mine = chain_weight(plans, L_in, Tb_in, Tt, dv.max_label, dv.log_domain);
    int before = 0, last_end = 0;
    for (int j = tid; j < B; j += kRowThreads) {
        const int Lj = dv.label_lengths[j], Tj = dv.input_lengths[j];
        const long long w = chain_weight(plans, Lj, Tj, Tt, dv.max_label, dv.log_domain);
        before += (w > mine || (w == mine && j < b)) ? 1 : 0;
        if (dv.tasks) last_end = max(last_end, chain_end_estimate(plans, Lj, Tj, Tt, dv.max_label, dv.log_domain));
    }
    if (before) atomicAdd(&s_rank, before);
    if (last_end) atomicMax(&s_last_end, last_end);
    __syncthreads();
    // (workers in the lattice launch: the utterances that end last are the gradient launch's, as in prepare)
    const bool later = dv.tasks && ends_late(chain_end_estimate(plans, L_in, Tb_in, Tt, dv.max_label, dv.log_domain),
                                             s_last_end, dv.share_percent);
    const bool invalid = bad_length || s_bad != 0;
    const int Tb = invalid ? 0 : Tb_in;
    const bool runs = !invalid && Tb > 0 && Tb >= L + s_repeats;
    const int Lp = invalid ? 0 : L;
    Utt m;
    m.Tb = Tb;
    m.L = Lp;
    m.lab_off = b * dv.max_label;
    m.flags = (runs ? kUttRuns : 0) | (invalid ? kUttInvalid : 0) |
              ((dv.log_domain || Tb > kLinearMaxFrames || tight_fit(Tb, L, s_repeats)) ? kUttLogDomain : 0) |
              (!invalid && plans.two_pairs(L) ? kUttTwoPairs : 0) | (later ? kUttGradientLater : 0);
    m.f_off = b * Tt;
    m.waves = plans.waves1(Lp);
    m.halo = plans.halo1(Lp);
    m.waves2 = plans.waves2(Lp);
    m.halo2 = plans.halo2(Lp);
    m.poll_budget = dv.poll_budget;
    m.e_direct = emission_layout(A);
    m.e_pitch = m.e_direct == kEmitSymbolMajor ? Tt : m.L;
    m.e_off = static_cast<int64_t>(b) * Tt * (m.e_direct ? A : dv.max_label);
    m.ab_off = static_cast<int64_t>(b) * Tt * lattice_pitch(dv.max_label);
    if (tid == 0) {
        dv.meta[b] = m;
        dv.status_words[b] = invalid ? 1 : 0;
        // heaviest first, in blocks of kChainBlock utterances: a block's forward chains, then its backward chains
        // Launches of more chains than compute units: workgroup i shares its compute unit with workgroups
        // i +- n_cu, so every other round of n_cu chains runs lightest first, and a compute unit's chains
        // add up to about the same (the host's order_chains goes by the SIMDs' loads; this is its first-order part).
        int rank = s_rank;
        const int per_round = dv.n_cu / dv.dirs;
        if (per_round >= kChainBlock && B * dv.dirs > dv.n_cu && ((rank / per_round) & 1)) {
            const int round_first = rank - rank % per_round, in_round = min(per_round, B - round_first);
            rank = round_first + (in_round - 1 - rank % per_round);
        }
        const int first = rank - rank % kChainBlock, in_block = min(kChainBlock, B - first);
        for (int d = 0; d < dv.dirs; ++d) dv.order[first * dv.dirs + d * in_block + rank % kChainBlock] = 2 * b + d;
    }
    return m;
}

template <typename T>
__global__ __launch_bounds__(kRowThreads)
void ctc_softmax_narrow_kernel(const T* __restrict__ x, const NarrowImage image, int* __restrict__ workspace_words,
                               float* __restrict__ lse, float* __restrict__ emit_blank,
                               float* __restrict__ emit_label, int* __restrict__ row_flags,
                               const SetupArgs sa, const NarrowArgs args, const NarrowDevice dv,
                               int Tt, int B, int A, int blank)
{
    constexpr int kRows = kFlagFrames, kPerRow = kRowThreads / kRows;
    static_assert(kPerRow == 4, "a quad per frame");
    extern __shared__ float lp[];                          // [kRows][A]
    __shared__ int s_lab[kSetupLabelSlots];
    __shared__ int s_small;
    const int b = blockIdx.y, tid = threadIdx.x;
    // (device-resident metadata with workers in the lattice launch: one more column, whose first workgroup
    // builds their task list)
    const int row_blocks = static_cast<int>(gridDim.x) - sa.parts - (dv.tasks ? 1 : 0);
    if (dv.tasks && blockIdx.x == gridDim.x - 1) {
        if (b == 0) build_task_table(dv, args.plans, Tt, B);
        return;
    }
    if (static_cast<int>(blockIdx.x) >= row_blocks && dv.labels) {
        // device-resident metadata: the first of these workgroups builds the record (and writes what depends on
        // it), the others group the label's positions, for which they need the label only: side by side, so that
        // the launch lasts as long as the longer of the two, not their sum
        const int part = static_cast<int>(blockIdx.x) - row_blocks;
        if (part == 0) {
            setup_words(build_record(dv, args.plans, b, Tt, B, A, blank), b, sa);
            return;
        }
        Utt m{};
        const int L = dv.label_lengths[b], Tb = dv.input_lengths[b];
        const bool bad_length = L < 0 || L > dv.max_label || Tb < 0 || Tb > Tt;
        m.L = bad_length ? 0 : L;
        m.lab_off = b * dv.max_label;
        setup_role(m, b, dv.labels, sa, s_lab, part - 1, sa.parts - 1, nullptr, nullptr, false);
        return;
    }
    if (static_cast<int>(blockIdx.x) >= row_blocks) {
        // (what the setup role uses of the utterance's record: no read of the record out of host memory,
        // so that the label's bytes are the first and only thing this workgroup waits for from there)
        Utt m{};
        m.Tb = args.rows.frames[b] & (kRowsGradientLater - 1);
        m.flags = ((args.rows.frames[b] & kRowsRun) ? kUttRuns : 0) |
                  ((args.rows.frames[b] & kRowsGradientLater) ? kUttGradientLater : 0);
        m.L = args.rows.label_length[b];
        m.lab_off = args.rows.labels_before[b];
        const int part = static_cast<int>(blockIdx.x) - row_blocks;
        // this workgroup's share of the image
        const int groups = B * sa.parts, group = b * sa.parts + part;
        const int share = (image.count + groups - 1) / groups;
        for (int i = group * share + tid; i < min((group + 1) * share, image.count); i += kRowThreads)
            if (i < image.labels_first || i >= image.labels_end) workspace_words[i] = image.words[i];
        setup_role(m, b, nullptr, sa, s_lab, part, sa.parts,
                   reinterpret_cast<const unsigned char*>(image.words) + image.labels8_offset, image.labels_out);
        return;
    }
    // (the fields of the utterance's record that the rows need)
    struct { int Tb, flags, f_off, e_pitch; int64_t e_off; } m;
    if (dv.labels) {
        // (whether an alignment exists is not known here: the rows of every utterance with frames are prepared)
        const int L = dv.label_lengths[b], Tb = dv.input_lengths[b];
        const bool bad_length = L < 0 || L > dv.max_label || Tb < 0 || Tb > Tt;
        m.Tb = bad_length ? 0 : Tb;
        m.flags = kUttRuns;
        m.f_off = b * Tt;
        m.e_pitch = Tt;
    } else {
        m.Tb = args.rows.frames[b] & (kRowsGradientLater - 1);
        m.flags = (args.rows.frames[b] & kRowsRun) ? kUttRuns : 0;
        m.f_off = args.rows.frames_before[b];
        m.e_pitch = m.Tb;
    }
    m.e_off = static_cast<int64_t>(m.f_off) * A;
    const int t0 = blockIdx.x * kRows;
    if (t0 >= m.Tb) return;
    if (tid == 0) s_small = 0;
    const int r = tid / kPerRow, q = tid % kPerRow, t = t0 + r;
    float* lrow = lp + r * A;
    if (t < m.Tb) {
        const T* row = x + (static_cast<size_t>(t) * B + b) * A;
        float mx = -__builtin_inff();
        // eight reads in flight per thread: a row costs a few memory latencies, not A / kPerRow
        for (int k0 = q; k0 < A; k0 += 8 * kPerRow) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int k = k0 + u * kPerRow;
                v[u] = (k < A) ? load_elem(row, k) : -__builtin_inff();
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int k = k0 + u * kPerRow;
                if (k < A) lrow[k] = v[u];
                mx = fmaxf(mx, v[u]);
            }
        }
        mx = quad_max(mx);
        float sum = 0.0f;
        for (int k = q; k < A; k += kPerRow) sum += fast_exp2((lrow[k] - mx) * kLog2e);
        sum = quad_sum(sum);
        const float ls = fast_log2(sum);
        const float l2 = fmaf(mx, kLog2e, ls);
        bool unused = false;       // (what counts is which of the coded emissions get stored below)
        for (int k = q; k < A; k += kPerRow) lrow[k] = encode_emission(log2_softmax(lrow[k], mx, ls), unused, sa.plain_logs);
        if (q == 0) lse[static_cast<size_t>(b) * Tt + t] = l2;
    }
    if (!(m.flags & kUttRuns)) return;
    __syncthreads();
    const int rows = min(kRows, m.Tb - t0);
    bool small = false;
    if (tid < rows) {
        const float e = lp[tid * A + blank];
        emit_blank[kBlankSlack + m.f_off + t0 + tid] = e;
        sa.emit_blank64[kBlankSlack + m.f_off + t0 + tid] = static_cast<double>(emission_probability(e));
        small = !sa.plain_logs && e < 0.0f;
    }
    // The emission block: a symbol's frames side by side, e_pitch floats per symbol (fetch_frames).
    // A wavefront writes up to 64 frames of one symbol at a time.
    float* out = emit_label + kLabelSlack + m.e_off + t0;
    const int rr = tid & 63;
    if (rr < rows)
        for (int a = tid >> 6; a < A; a += kRowThreads / 64) {
            const float e = lp[rr * A + a];
            out[static_cast<size_t>(a) * m.e_pitch + rr] = e;
            small = small || (!sa.plain_logs && e < 0.0f);
        }
    if (small) s_small = 1;
    __syncthreads();
    if (tid == 0) row_flags[static_cast<size_t>(b) * row_blocks + blockIdx.x] = s_small;
}

// Has the narrow softmax launch met an emission below the linear domain's range in one of the
// utterance's frames?  Asked by a whole wavefront; the same answer in every lane.
__device__ __forceinline__ bool rows_flagged(const int* __restrict__ row_flags, int b, int blocks_per_utterance, int Tb)
{
    if (!row_flags) return false;
    const int lane = threadIdx.x & 63, n = (Tb + kFlagFrames - 1) / kFlagFrames;
    bool any = false;
    for (int i = lane; i < n; i += 64) any = any || row_flags[static_cast<size_t>(b) * blocks_per_utterance + i] != 0;
    return __ballot(any) != 0;
}

// ---- lattice storage -------------------------------------------------------------------------
// What the recursions leave for the gradient, per label state, frame and direction: a number
// m * 2^e, as
//   a value word (uint32): the high dword of the fp64 m (sign, exponent, top 20 mantissa bits),
//                          one per state and frame, rows of lattice_pitch(L) words by frame;
//   an exponent word (int32): e, one per state and exponent row.
// A linear-domain chain stores its state in the lane's frame as it stands (no arithmetic on the
// way out), and the frame changes only when a chunk ends: it writes one exponent row per chunk
// (exponent_row), 4.5 bytes per state and frame in all.  A log-domain chain has a new exponent at
// every step and writes one exponent row per step.  Both blocks of a direction are sized for the
// latter (which chain runs is decided on the GPU, by the softmax launch): values in the first
// half of the direction's region, exponents in the second.
// Twenty mantissa bits bound the relative error of a state's share alpha * beta / p by 2^-19,
// which is 2e-6 of a gradient entry at most.  Exponents stay above -2^30 so that the sum of two
// cannot wrap.
// The mass p of an utterance (its reciprocal) keeps both parts in one 8-byte word (pack_state).
__device__ __forceinline__ double pack_state(double in_frame, int frame)
{
    return __hiloint2double(__double2hiint(in_frame), frame);
}
// Loads of what a chain has left for the gradient.  The gradient launch reads plainly.  A worker
// of the lattice launch (gradient_worker) reads while other chains still run: its loads carry
// device scope, so that the compute unit's own cache, which may hold a line from before the chain
// wrote it, is passed by and the L2 answers, which chain and worker share (see gradient_worker).
template <bool kCoherent, typename W>
__device__ __forceinline__ W lattice_load(const W* p)
{
    if (kCoherent) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return *p;
}
template <typename W>
__device__ __forceinline__ void lattice_store(W* p, W v) { *p = v; }

// Exponent row of the state a chain reached at its step `step` (0 .. Tb-1; a forward chain's step
// is the frame, a backward chain's Tb-1-frame).  Linear domain: the initial frame serves step 0 and
// the first chunk (steps 1 .. kChunk), each later chunk has a row of its own.
__device__ __forceinline__ int exponent_row(int step, bool log_domain)
{
    return log_domain ? step : (max(step - 1, 0) / kChunk);
}
// A base-2 logarithm (log-domain chains) as value and exponent: m = 2^fraction in [1, 2), e = floor.
// log 0 (and anything as small) is stored as the number 0.
__device__ __forceinline__ void split_log2(double w, uint32_t& value, int& exponent)
{
    const double whole = floor(w);
    const double m = static_cast<double>(fast_exp2(static_cast<float>(w - whole)));
    const bool real = w > -1.0e9 && w < 1.0e9;
    value = real ? static_cast<uint32_t>(__double2hiint(m)) : 0u;
    exponent = real ? static_cast<int>(whole) : 0;
}
__device__ __forceinline__ double pack_log2(double w)          // the same as one word (1 / p)
{
    uint32_t value;
    int exponent;
    split_log2(w, value, exponent);
    return __hiloint2double(static_cast<int>(value), exponent);
}
// alpha * beta * (1 / p) from the stored parts.  (The missing low dword of a value is a relative
// 2^-20 at most.)  Either of alpha and beta may lie a thousand binary orders below or above the unit
// of its own frame (lane_frame) while their product is a share of order one, so the factors are
// balanced before they are multiplied.
__device__ __forceinline__ float mass_share(uint32_t a_value, int a_exponent, uint32_t b_value, int b_exponent,
                                            float inverse_p_mantissa, int inverse_p_exponent)
{
    // alpha's word is brought to [1, 2) by its own exponent field, and everything else goes to beta: the
    // product is a share, at most 1, so beta's factor stays in range wherever alpha is not 0; next to an
    // alpha that is the number 0 it is capped, so that the product is 0 and not 0 times infinity.
    const int to_one = 1023 - static_cast<int>(a_value >> 20);
    const int rest = a_exponent + b_exponent + inverse_p_exponent - to_one;
    const double a = __hiloint2double(static_cast<int>(a_value), 0);
    const double b = __hiloint2double(static_cast<int>(b_value), 0);
    return static_cast<float>(__builtin_amdgcn_ldexp(a, to_one) * fmin(__builtin_amdgcn_ldexp(b, rest), 0x1p200)) *
           inverse_p_mantissa;
}

// ---- lattice recursions ------------------------------------------------------------------
// log2(2^a + 2^b) for fp64 a, b with the exponentials taken on the fp32 difference.
__device__ __forceinline__ double lse2(double a, double b)
{
    const double hi = fmax(a, b);
    const float d = static_cast<float>(a - b);
    return hi + static_cast<double>(fast_log2(1.0f + fast_exp2(-fabsf(d))));
}
// Lane i receives the value of lane i-1 (DPP wave_shr:1).  The shift writes nothing into lane 0,
// which therefore keeps what `into` held there: initialised once to log 0 and passed back in at
// every step, it needs no refill (two moves per step otherwise).
__device__ __forceinline__ double shift_up(double v, int& into_lo, int& into_hi)
{
    into_lo = __builtin_amdgcn_update_dpp(into_lo, __double2loint(v), 0x138, 0xf, 0xf, false);
    into_hi = __builtin_amdgcn_update_dpp(into_hi, __double2hiint(v), 0x138, 0xf, 0xf, false);
    return __hiloint2double(into_hi, into_lo);
}

// max(window of the lane below, mine) in one instruction, the DPP shift as an operand of the maximum.
// Lane 0 has no lane below: the instruction then leaves its register alone, and `window` starts out as
// the lanes' own values.  (s_nop 1: a DPP operand must be two wait states old.)
__device__ __forceinline__ int window_max_step(int window, int mine)
{
    asm("s_nop 1\n\tv_max_i32_dpp %0, %0, %1 wave_shr:1 row_mask:0xf bank_mask:0xf" : "+v"(window) : "v"(mine));
    return window;
}

constexpr int kHaloEntries = 64;      // 16-byte entries of one wavefront boundary's exchange buffer (2 x 32)

enum class Sync { kNone, kHalo, kBarrier };

// Predecessor choices of a pair at one frame, as stored for the backtrace; each field is the
// number of states the walk moves down.  Bits 2..3, the label state: 0 = stayed, 1 = came from
// the pair's blank, 2 = came from the label of the pair before (skipping the blank).  Bit 0, the
// blank state: 0 = stayed, 1 = came from the label of the pair before.
// The next kChunk frames of one symbol out of a transposed emission block (symbol-major: a
// symbol's frames lie side by side), in the order the chain takes them, in two 16-byte loads
// instead of kChunk loads a row apart.  `p` points at the frame of the step before the first one
// wanted and moves on by `advance` floats (kChunk in the chain's direction; 0 for a lane
// without a label state, which keeps reading its constants).
struct __attribute__((packed, aligned(4))) Float4 { float v[4]; };
static_assert(kChunk == 8, "fetch_frames loads two Float4");
template <bool kBackward>
__device__ __forceinline__ void fetch_frames(const float*& p, int advance, float (&el)[kChunk])
{
    const Float4 lo = *reinterpret_cast<const Float4*>(p + fetch_window_first(kBackward));
    const Float4 hi = *reinterpret_cast<const Float4*>(p + fetch_window_first(kBackward) + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        el[i] = kBackward ? hi.v[3 - i] : lo.v[i];
        el[4 + i] = kBackward ? lo.v[3 - i] : hi.v[i];
    }
    p += advance;
}
constexpr int kFromSame = 0, kFromBlank = 1 << 2, kFromPrevLabel = 2 << 2, kBlankFromPrevLabel = 1;

// LDS of a chain's workgroup (dynamic, sized by the launch for its widest chain): a header, then
// one block per wavefront that holds what that wavefront hands to the one above it.
struct HaloHeader {
    // Cost-only chains: the last wavefront to finish writes the cost (or NaN if any gave up).
    int finished;                     // wavefronts that have reached the end of the chain
    int gave_up;
    float cost;
    int unused;
};
// Chains with one pair per lane.
struct HaloWave {
    double2 data[kHaloEntries];
    int frame[kHaloEntries];          // linear-domain chains: the frame exponent that goes with each entry
    int ready;                        // last generation this wavefront has published
    int done;                         // last generation this wavefront has taken from the one below
    int unused[2];
};

// Chains with two pairs per lane (run_chain_linear2).
constexpr int kRing = 4;                  // hand-overs a boundary's buffer holds
constexpr int kHalo2Lanes = 16;           // most halo lanes plan_waves2 asks for
struct Halo2Wave {
    double2 data[kRing][kHalo2Lanes][2];      // [hand-over mod kRing][halo lane][pair]: (blank, label)
    int2 tag[kRing][kHalo2Lanes];             // (the lane's frame, number of the hand-over)
};
constexpr size_t kHaloWaveBytes = sizeof(HaloWave) > sizeof(Halo2Wave) ? sizeof(HaloWave) : sizeof(Halo2Wave);
static_assert(sizeof(HaloHeader) % 16 == 0 && kHaloWaveBytes % 16 == 0, "the blocks hold 16-byte entries");
// Bytes of dynamic LDS of a lattice launch whose workgroups have `waves` wavefronts.
constexpr size_t halo_lds_bytes(int waves) { return sizeof(HaloHeader) + static_cast<size_t>(waves) * kHaloWaveBytes; }
template <typename Wave>
__device__ __forceinline__ Wave* halo_wave(void* lds, int wave)
{
    return reinterpret_cast<Wave*>(static_cast<char*>(lds) + sizeof(HaloHeader) + static_cast<size_t>(wave) * kHaloWaveBytes);
}


// One chain = one direction of one utterance.  A lane owns the pair
//   forward : (blank state 2j,       label j        = state 2j+1)
//   backward: (blank state 2(L-j),   label L-1-j    = state 2(L-j)-1)
// so that in both directions the only value needed from a neighbour is the label entry of
// pair j-1 (one DPP shift), and both directions run the same recursion on the "inclusive"
// quantity
//   w_step(state) = E_frame(state) + log2 sum over predecessors of 2^w_{step-1}
// which is alpha going forward.  Going backward, the sum before E is added is the beta that
// excludes its own frame's emission, and that is what gets stored, so that
// log alpha + log beta is the log mass of alignments through a state.
//
// Storage: only the label states are written, alpha_row[1 + i] = alpha(2i+1), beta_row[1 + i] =
// beta(2i+1), row pitch L+2 words (lattice_pitch; the first and the last column stay unused).  The blank states are needed by the recursion but not by
// the gradient, which takes the blank's occupancy as 1 minus that of all label states
// (sum_s alpha_t(s) beta_t(s) = p at every frame).
//
// A lone wavefront on its SIMD issues an instruction about every five clocks whatever its kind
// (a vector memory instruction counts for three), so the step is written for instruction count:
// pointers advance by adds, lanes without a pair write to a sink, whole chunks run without a look
// at the step number.
//
// Labels of more than 63 symbols span several wavefronts.  Exchanging a value at every step
// costs more than a third of the step, so with Sync::kHalo each wavefront recomputes, in its
// first `halo` lanes, the last `halo` pairs of the wavefront below it:
//     pair of (wave, lane) = wave * (64 - halo) + lane
// (wavefront 0 has nothing below it: all its 64 lanes are exact, its lane 0 is pair 0).
// An error at lane 0 (whose neighbour is missing) moves up one lane per step, so the lanes
// from `halo` on stay exact for `halo` steps.  Every `halo` steps (a whole number of chunks)
// the lower wavefront hands
// over the exact state of those pairs through LDS (a small ring per boundary, guarded by two
// counters: `ready` written by the producer after the data, `done` by the consumer after its
// read).  No barrier; the wavefronts run skewed.  A wavefront waits for data only on lower
// ones and for space only on higher ones, wavefront 0 needs no data and the last one no space,
// so every wait ends; a poll budget bounds them regardless and raises chain_err when spent.
template <bool kBackward, Sync kSync, Mode kMode, bool kSymbolMajor>
__device__ __forceinline__ void run_chain_log(const Utt m, const int u, const int* __restrict__ labels,
                                          const float* __restrict__ emit_blank,
                                          const float* __restrict__ emit_label,
                                          uint32_t* __restrict__ out, int* __restrict__ out_exponents,
                                          double* __restrict__ logp,
                                          float* __restrict__ costs, int* __restrict__ chain_err,
                                          uint32_t* __restrict__ sink, void* lds)
{
    static_assert(kMode == Mode::kGrad || !kBackward, "only the gradient needs the backward chain");
    // Launches for the most probable alignment store plain logarithms, the others coded emissions.
    constexpr bool kCoded = kMode != Mode::kBest;
    const int L = m.L, Tb = m.Tb, P = L + 1;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // (uniform: in a scalar register)
    const int halo = (kSync == Sync::kHalo) ? m.halo : 0;
    const int j = wave * (64 - halo) + lane;
    const int* lab = labels + m.lab_off;
    const bool has_label = j >= 0 && j < L;
    const bool active = (wave == 0 || lane >= halo) && j <= L;   // this lane stores pair j
    const int li = kBackward ? (L - 1 - j) : j;          // label index of this pair's label state
    // May the label state be entered from pair j-1's label?  (Not across equal symbols.)
    const bool skip_ok = has_label && j >= 1 && lab[li] != lab[kBackward ? (li + 1) : (li - 1)];
    const double skip_penalty = skip_ok ? 0.0 : kNeg;

    // Frame of step s: s going forward, Tb-1-s going backward.
    const int f0 = kBackward ? (Tb - 1) : 0;
    const int fdir = kBackward ? -1 : 1;
    // Label emissions: a per-lane pointer that moves one row per step.  A lane without a label
    // state reads a constant log 0 and stays there.
    // (In a symbol-major block the pointer moves one float per step: emission_layout.  The layout
    // is the launch's, a template parameter: a test at run time would join two paths with
    // different numbers of loads under way, and the waits after the join would be the
    // cautious ones.)
    constexpr bool direct = kSymbolMajor;
    const float* ep = emit_label + label_emission_offset(m, has_label, direct, has_label ? lab[li] : 0, li, f0, kLogZeroEmission);
    const int64_t estride = label_emission_step(m, has_label, false, fdir);
    const int eadvance = static_cast<int>(label_emission_step(m, has_label, true, fdir)) * kChunk;
    // Blank emissions: lane i of a chunk's load takes the frame of step (chunk start + i % kChunk).
    const float* bp = emit_blank + blank_emission_offset(m, f0, fdir, lane);
    // Output: only the label state of each pair is kept (row pitch L+2 words, column = 1 + label
    // index, in both directions; value rows by frame, exponent rows by step: one per step in the
    // log domain); the gradient gets the blank's share as the complement.
    // Lanes that store nothing write to a sink instead.
    // With Mode::kBest the value block holds one byte per pair and frame instead (row pitch
    // L+1 bytes, column = pair), pair L included: its blank state has a choice to record.
    constexpr int64_t kOutBytes = (kMode == Mode::kBest) ? 1 : 4;
    const int64_t out_pitch = (kMode == Mode::kBest) ? P : lattice_pitch(L);
    const bool stores = (kMode == Mode::kBest) ? active : (active && has_label);
    char* op = stores ? reinterpret_cast<char*>(out) +
                            (m.ab_off + static_cast<int64_t>(f0) * out_pitch + (kMode == Mode::kBest ? j : li + 1)) * kOutBytes
                      : reinterpret_cast<char*>(sink);
    const int64_t ostride = stores ? static_cast<int64_t>(fdir) * out_pitch * kOutBytes : 0;
    int* xp = (stores && kMode == Mode::kGrad) ? out_exponents + m.ab_off + li + 1 : reinterpret_cast<int*>(sink);
    const int64_t xstride = (stores && kMode == Mode::kGrad) ? out_pitch : 0;
    int choice = 0;
    auto store_state = [&](double w) {
        uint32_t value;
        int exponent;
        split_log2(w, value, exponent);
        lattice_store(reinterpret_cast<uint32_t*>(op), value);
        lattice_store(xp, exponent);
        xp += xstride;
    };

    HaloHeader* const hl = static_cast<HaloHeader*>(lds);
    const int last_wave = m.waves - 1;
    HaloWave* const mine_lds = halo_wave<HaloWave>(lds, wave);
    HaloWave* const below_lds = halo_wave<HaloWave>(lds, wave > 0 ? wave - 1 : 0);
    HaloWave* const above_lds = halo_wave<HaloWave>(lds, wave < last_wave ? wave + 1 : wave);
    int budget = m.poll_budget;                          // polls left before this wavefront gives up waiting
    bool lost = false;                                   // it did give up: what it computed since is not to be trusted
    // Hand-overs fall on chunk boundaries (the halo is a multiple of kChunk), so the step
    // itself carries no countdown and the hand-over code exists once per chunk, not per step.
    const int chunks_per_hand_over = halo / kChunk;
    int until_hand_over = chunks_per_hand_over;          // chunks until the next hand-over
    int generation = 0;
    // Each boundary's buffer is used as two halves of 32 entries, alternating by generation
    // (halo <= 32), so a producer may run one hand-over ahead of its consumer.
    int half = 0;                                        // entry offset of the half in use: 0 or 32
    double2* const wr_base = (kSync == Sync::kHalo)
        ? &mine_lds->data[lane >= 64 - halo ? lane - (64 - halo) : 0] : nullptr;
    const double2* const rd_base = (kSync == Sync::kHalo)
        ? &below_lds->data[lane < halo ? lane : 0] : nullptr;
    int* const my_ready = &mine_lds->ready;
    int* const my_done = &mine_lds->done;
    int* const up_done = &above_lds->done;
    int* const low_ready = &below_lds->ready;

    double i_blank = (j == 0) ? 0.0 : kNeg;
    double i_label = (j == 0 && has_label) ? 0.0 : kNeg;
    double v_blank, v_label;

    auto counter = [&](int* p) {
        return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    auto uniform = [](int v) { return __builtin_amdgcn_readfirstlane(v); };
    int done_seen = 0;                                   // a (possibly old) reading of done[wave + 1]
    // After a step whose number is a multiple of `halo`: pass the exact state of the top `halo`
    // pairs up, take the exact state of the halo pairs from below.
    auto hand_over = [&]() {
        ++generation;
        half ^= 32;
        if (wave < last_wave) {
            // Space: the consumer must have taken generation - 2.  The reading from the last
            // hand-over usually shows that already.
            int seen = uniform(done_seen);
            if (__builtin_expect(seen < generation - 2, 0)) {
                while (seen < generation - 2 && budget > 0) {
                    --budget;
                    seen = uniform(counter(up_done));
                }
                lost = lost || seen < generation - 2;
            }
            if (lane >= 64 - halo) wr_base[half] = make_double2(v_blank, v_label);
            // LDS operations of a wavefront complete in order: the counter follows the data.
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            if (lane == 63) __hip_atomic_store(my_ready, generation, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            done_seen = counter(up_done);                // consumed at the next hand-over
        }
        if (wave > 0) {
            // Counter and data are read back to back; the data count only if the counter,
            // read first, already showed this generation.
            int ready = counter(low_ready);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            double2 v = rd_base[half];
            ready = uniform(ready);
            if (__builtin_expect(ready < generation, 0)) {
                while (ready < generation && budget > 0) {
                    --budget;
                    ready = counter(low_ready);
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    v = rd_base[half];
                    ready = uniform(ready);
                }
                lost = lost || ready < generation;
            }
            if (lane < halo) {
                v_blank = v.x;
                v_label = v.y;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            if (lane == 0) __hip_atomic_store(my_done, generation, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    };

    // Label value of pair j-1 after step s (log 0 for pair 0).  `mine` is this lane's.
    int prev_lo = __double2loint(kNeg), prev_hi = __double2hiint(kNeg);
    auto from_prev_pair = [&](double mine, int s) {
        double r = shift_up(mine, prev_lo, prev_hi);
        if (kSync == Sync::kBarrier) {
            double (*xch)[16] = static_cast<double (*)[16]>(lds);
            if (lane == 63) xch[s & 1][wave] = mine;
            __syncthreads();
            if (lane == 0 && wave > 0) r = xch[s & 1][wave - 1];
        }
        return r;
    };

    auto finish_step = [&](double eb, float el) {
        v_blank = i_blank + eb;
        v_label = i_label + (kCoded ? emission_log2(el) : static_cast<double>(el));
        if (kMode == Mode::kBest) {
            *op = static_cast<unsigned char>(choice);
        } else if (kMode == Mode::kLoss) {
            // nothing is kept
        } else {
            store_state(kBackward ? i_label : v_label);
        }
        op += ostride;
    };
    // After the last step of a chunk (the last chunk of a chain may be short: its hand-over
    // then comes early, which every wavefront of the chain does alike).
    auto end_chunk = [&]() {
        if (kSync == Sync::kHalo) {
            if (--until_hand_over == 0) {
                hand_over();
                until_hand_over = chunks_per_hand_over;
            }
        }
    };
    auto advance = [&](int step, double eb, float el) {
        const double prev = from_prev_pair(v_label, step - 1);
        if (kMode == Mode::kBest) {
            const double via_skip = prev + skip_penalty;
            const bool blank_moves = prev > v_blank;
            i_blank = blank_moves ? prev : v_blank;
            double best = v_label;
            choice = kFromSame;
            if (v_blank > best) { best = v_blank; choice = kFromBlank; }
            if (via_skip > best) { best = via_skip; choice = kFromPrevLabel; }
            i_label = best;
            choice |= blank_moves ? kBlankFromPrevLabel : 0;
        } else {
            // The blank state sums its own value and the label of the pair before; where the
            // label state may also be entered from that label (skip), its three-term sum is
            // its own value plus exactly the blank state's new sum, else plus the old blank:
            // two two-term sums per pair instead of a two- and a three-term one.
            i_blank = lse2(v_blank, prev);
            i_label = lse2(v_label, skip_ok ? i_blank : v_blank);
        }
        finish_step(eb, el);
    };
    auto readlane = [](float v, int l) {
        return __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(v), l));
    };

    // step 0: every lane starts from the exact state of its pair, halo lanes included
    {
        const Log2Parts ebv = kCoded ? emission_log2_parts(*bp) : Log2Parts{*bp, 0.0f};
        v_blank = i_blank + static_cast<double>(readlane(ebv.whole, 0)) + static_cast<double>(readlane(ebv.part, 0));
        v_label = i_label + (kCoded ? emission_log2(*ep) : static_cast<double>(*ep));
        // (the predecessor choices of frame 0 are never looked at: nothing is written for it)
        if (kMode == Mode::kGrad) store_state(kBackward ? i_label : v_label);
        op += ostride;
    }

    // Emissions of steps 1..: two register sets, one in use, one being filled.
    float el_a[kChunk], el_b[kChunk], eb_a, eb_b;
    auto fetch = [&](float (&el)[kChunk], float& eb, int s0) {
        eb = bp[fdir * s0];
        if (direct) {
            fetch_frames<kBackward>(ep, eadvance, el);
            return;
        }
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            ep += estride;
            el[i] = *ep;
        }
    };
    // One copy of the step per chunk position and register set: the kernel has to stay well
    // inside the instruction cache that two compute units share.
    // Whole chunks run without looking at the step number; only the last, short chunk of a
    // chain checks every step against the end.
    auto run = [&](const float (&el)[kChunk], const float eb_coded, int s0, bool whole) {
        const Log2Parts eb = kCoded ? emission_log2_parts(eb_coded) : Log2Parts{eb_coded, 0.0f};
        auto blank_of_step = [&](int i) {
            const double whole_part = static_cast<double>(readlane(eb.whole, i));
            return kCoded ? whole_part + static_cast<double>(readlane(eb.part, i)) : whole_part;
        };
        if (whole) {
#pragma unroll
            for (int i = 0; i < kChunk; ++i) advance(s0 + i, blank_of_step(i), el[i]);
        } else {
#pragma unroll
            for (int i = 0; i < kChunk; ++i)
                if (s0 + i < Tb) advance(s0 + i, blank_of_step(i), el[i]);
        }
    };
    chain_schedule(Tb, [&](int s0) { fetch(el_a, eb_a, s0); __builtin_amdgcn_sched_barrier(0); },
                   [&](int s0) { fetch(el_b, eb_b, s0); __builtin_amdgcn_sched_barrier(0); },
                   [&](int s0, bool whole) { run(el_a, eb_a, s0, whole); }, [&](int s0, bool whole) { run(el_b, eb_b, s0, whole); },
                   end_chunk);

    if (!kBackward) {
        // p = alpha_{T-1}(2L) + alpha_{T-1}(2L-1): the blank of pair L and the label of pair L-1.
        // Pair L sits in an exact lane, and so does the lane below it or, if that is the last
        // halo lane, it is still exact: the error from lane 0 needs `halo` steps to get there,
        // and a hand-over that fell due after the last step has been done by end_chunk.
        const double prev = from_prev_pair(v_label, Tb - 1);
        if (active && j == L) {
            if (kMode == Mode::kBest) {
                // the better of the two end states; logp carries which one to the backtrace
                const bool ends_on_label = prev > v_blank;
                const double lp = ends_on_label ? prev : v_blank;
                logp[u] = static_cast<double>(2 * L - (ends_on_label ? 1 : 0));
                costs[u] = (lp < -1.0e29) ? __builtin_inff() : static_cast<float>(-lp * kLn2);
            } else {
                const double lp = lse2(v_blank, prev);
                lattice_store(&logp[u], pack_log2(-lp));          // 1 / p
                const float cost = (lp < -1.0e29) ? __builtin_inff() : static_cast<float>(-lp * kLn2);
                if (kSync == Sync::kHalo && kMode == Mode::kLoss) hl->cost = cost;
                else costs[u] = cost;
            }
        }
    }
    if (kSync == Sync::kHalo && kMode == Mode::kLoss) {
        // No kernel follows that could turn a lost exchange into a NaN cost, so the cost is
        // written by whichever wavefront finishes last, once it has seen whether any gave up.
        // (One wavefront's LDS operations complete in order: flag and cost precede its count.)
        if (lost && lane == 0) hl->gave_up = 1;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        int before = 0;
        if (lane == 0)
            before = __hip_atomic_fetch_add(&hl->finished, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        before = __builtin_amdgcn_readfirstlane(before);
        if (before == m.waves - 1 && lane == 0) {
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int lost = __hip_atomic_load(&hl->gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            const float cost = hl->cost;
            costs[u] = lost ? __uint_as_float(0x7FC00000u) : cost;
        }
    } else if (kSync == Sync::kHalo && lost && lane == 0) {
        lattice_store(&chain_err[u], 1);
    }
}

// The same chain on probabilities instead of their logarithms: a step is then two fused
// multiply-adds, an addition and two multiplications per pair, a third of the instructions of the
// log-domain step and no transcendentals.  What makes it safe is an exponent per lane:
//   true value = (v_blank, v_label) * 2^frame
// with fp64 values and an int32 `frame` that is renewed after every chunk of kChunk steps:
//   frame = largest binary exponent among this pair and the kChunk pairs below it.
// Mass moves up by at most one pair per step, so until the next renewal everything that can
// reach the pair is at most 2^(kChunk+1) in its frame (no overflow), and its own mass cannot
// shrink by more than kChunk emissions, each at least 2^kLinearMinLog2, that is 800 of fp64's
// 1022 binary orders of magnitude (utterances with smaller emissions run the log-domain chain).
// Only what lies more than about 2^-1000 below the largest of its nine-pair window is rounded
// away.  The value shifted in from the pair below is brought into this lane's frame by `scale`
// = 2^(frame below - frame here), constant between renewals and folded into the multiply-adds.
//
// Storage (Mode::kGrad): the label state's value word at every step, its frame once per chunk
// (see "lattice storage").
constexpr int kNoExponent = -(1 << 28);   // exponent of zero: below every real one, far from int32's ends
// A lane's new frame is the largest exponent of its window (its own pairs and those that can reach it
// before the next renewal), so that nothing arriving overflows -- but no more than kFrameSlack above
// its own largest value where the window's top lies further up than that, down to kFrameDrop below the
// window's top.  With the window's top as the frame of every lane, a pair whose neighbours below carry
// 2^1000 times its mass was rounded away: wrong when those neighbours' mass can no longer reach the
// end of the label and the small pair is all there is (an utterance with exactly as many frames as its
// label needs, logits spread over 40 nats: cost off by 0.03, gradient by 0.03).  Now a pair keeps
// 2^-kFrameSlack of its frame, 2^-(kFrameSlack + 800) after a chunk of the smallest emissions the
// linear domain admits, as long as the window's top is within 2^(kFrameSlack + kFrameDrop) of it; what
// arrives from the window is at most 2^(kFrameDrop + 9) in the lane's frame, and two neighbouring
// frames differ by at most kFrameSlack + kFrameDrop, which the factor between them (scale) can hold.
// A pair further below its window than that has neighbours with 2^950 times its mass that can still
// reach the end (utterances with fewer than kTightFrames frames to spare, where they could not, run in
// the log domain from the start: tight_fit), each of their extra moves costing an emission of 2^-100 at
// worst: what is rounded away then is below 2^-50 of the whole.
constexpr int kFrameSlack = 150, kFrameDrop = 800;
// (A lane without mass, whose own largest exponent is kNoExponent, sits kFrameDrop below the top: the
// first mass to reach it may come from a lane whose own frame lies that low, and must not be rounded
// away on arrival.)
__device__ __forceinline__ int lane_frame(int window_top, int own_top)
{
    return window_top - min(max(window_top - own_top - kFrameSlack, 0), kFrameDrop);
}
// A renewal is put off while it is not needed (a third of a chunk's instructions are the renewal's): every
// pair of the wavefront has mass, lies within [2^kEasyLow, 2^kEasyHigh] of its frame, and at the last
// renewal no frame lay more than kSmoothFrames below the frame of the lane below it.  Then one more chunk
// takes a value down to 2^(kEasyLow - 800) at worst, and up to 3^kChunk times the largest of the nine-pair
// window in this lane's frame, 2^(kEasyHigh + kChunk * kSmoothFrames + 13): both far inside fp64.  The
// frames, the scale factors and the exponent rows simply stay what they are.
constexpr int kEasyLow = -200, kEasyHigh = 100;
constexpr int kSmoothFrames = 60;
// The test, on the high dword of the largest value of a lane (biased exponent in bits 20..30): one
// subtraction and one unsigned compare; zero, denormals, infinities and NaN fail it.
__device__ __forceinline__ bool outside_easy_range(double top)
{
    const unsigned hi = static_cast<unsigned>(__double2hiint(top));
    return hi - (static_cast<unsigned>(1023 + kEasyLow) << 20) >= (static_cast<unsigned>(kEasyHigh - kEasyLow + 1) << 20);
}

template <bool kBackward, Sync kSync, Mode kMode, bool kSymbolMajor>
__device__ __forceinline__ void run_chain_linear(const Utt m, const int u, const int* __restrict__ labels,
                                                 const float* __restrict__ emit_blank,
                                                 const double* __restrict__ emit_blank64,
                                                 const float* __restrict__ emit_label,
                                                 uint32_t* __restrict__ out, int* __restrict__ out_exponents,
                                                 double* __restrict__ logp,
                                                 float* __restrict__ costs, int* __restrict__ chain_err,
                                                 uint32_t* __restrict__ sink, void* lds)
{
    static_assert(kMode == Mode::kGrad || !kBackward, "only the gradient needs the backward chain");
    static_assert(kSync != Sync::kBarrier, "the barrier kernel runs the log-domain chain");
    static_assert(kMode != Mode::kBest, "the maximum recursion runs in the log domain");
    const int L = m.L, Tb = m.Tb;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // (uniform: in a scalar register)
    const int halo = (kSync == Sync::kHalo) ? m.halo : 0;
    const int j = wave * (64 - halo) + lane;             // pair of this lane (see run_chain_log)
    const int* lab = labels + m.lab_off;
    const bool has_label = j >= 0 && j < L;
    const bool active = (wave == 0 || lane >= halo) && j <= L;
    const int li = kBackward ? (L - 1 - j) : j;
    const bool skip_ok = has_label && j >= 1 && lab[li] != lab[kBackward ? (li + 1) : (li - 1)];

    const int f0 = kBackward ? (Tb - 1) : 0;
    const int fdir = kBackward ? -1 : 1;
    // A lane without a label state reads a constant probability 0 and stays there.
    constexpr bool direct = kSymbolMajor;                // see run_chain_log
    const float* ep = emit_label + label_emission_offset(m, has_label, direct, has_label ? lab[li] : 0, li, f0, kZeroEmission);
    const int64_t estride = label_emission_step(m, has_label, false, fdir);
    const int eadvance = static_cast<int>(label_emission_step(m, has_label, true, fdir)) * kChunk;
    // The blank's probability is the same for all lanes: an fp64 scalar, a chunk's frames in one load.
    (void)emit_blank;
    const double* const bq = emit_blank64;
    auto blank_window = [&](int s0) { return bq + blank64_window(m, f0, fdir, s0); };
    auto blank_of = [&](const double* w, int i) { return w[kBackward ? kChunk - 1 - i : i]; };
    // Values by frame, exponents by chunk (exponent_row): the lane's frame is what it is until the
    // chunk ends.
    const bool stores = kMode == Mode::kGrad && active && has_label;
    uint32_t* op = stores ? out + m.ab_off + static_cast<int64_t>(f0) * lattice_pitch(L) + li + 1 : sink;
    const int64_t ostride = stores ? static_cast<int64_t>(fdir) * lattice_pitch(L) : 0;
    int* xp = stores ? out_exponents + m.ab_off + li + 1 : reinterpret_cast<int*>(sink);
    const int64_t xstride = stores ? lattice_pitch(L) : 0;

    HaloHeader* const hl = static_cast<HaloHeader*>(lds);
    const int last_wave = m.waves - 1;
    HaloWave* const mine_lds = halo_wave<HaloWave>(lds, wave);
    HaloWave* const below_lds = halo_wave<HaloWave>(lds, wave > 0 ? wave - 1 : 0);
    HaloWave* const above_lds = halo_wave<HaloWave>(lds, wave < last_wave ? wave + 1 : wave);
    int budget = m.poll_budget;
    bool lost = false;
    const int chunks_per_hand_over = halo / kChunk;
    int until_hand_over = chunks_per_hand_over;
    int generation = 0;
    int half = 0;
    const int wr_slot = lane >= 64 - halo ? lane - (64 - halo) : 0;
    const int rd_slot = lane < halo ? lane : 0;
    double2* const wr_base = (kSync == Sync::kHalo) ? &mine_lds->data[wr_slot] : nullptr;
    const double2* const rd_base = (kSync == Sync::kHalo) ? &below_lds->data[rd_slot] : nullptr;
    int* const wr_frame = (kSync == Sync::kHalo) ? &mine_lds->frame[wr_slot] : nullptr;
    const int* const rd_frame = (kSync == Sync::kHalo) ? &below_lds->frame[rd_slot] : nullptr;
    int* const my_ready = &mine_lds->ready;
    int* const my_done = &mine_lds->done;
    int* const up_done = &above_lds->done;
    int* const low_ready = &below_lds->ready;

    double i_blank = (j == 0) ? 1.0 : 0.0;
    double i_label = (j == 0 && has_label) ? 1.0 : 0.0;
    double v_blank, v_label;
    int frame = 0;
    double scale = 1.0;                                  // 2^(frame of the pair below - frame)
    double skip_scale = skip_ok ? 1.0 : 0.0;             // the same where the label may be entered from that pair's label

    auto counter = [&](int* p) {
        return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    auto uniform = [](int v) { return __builtin_amdgcn_readfirstlane(v); };
    int done_seen = 0;
    // The exchange protocol of run_chain_log; an entry carries the pair's frame as well.
    auto hand_over = [&]() {
        ++generation;
        half ^= 32;
        if (wave < last_wave) {
            int seen = uniform(done_seen);
            if (__builtin_expect(seen < generation - 2, 0)) {
                while (seen < generation - 2 && budget > 0) {
                    --budget;
                    seen = uniform(counter(up_done));
                }
                lost = lost || seen < generation - 2;
            }
            if (lane >= 64 - halo) {
                wr_base[half] = make_double2(v_blank, v_label);
                wr_frame[half] = frame;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            if (lane == 63) __hip_atomic_store(my_ready, generation, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            done_seen = counter(up_done);
        }
        if (wave > 0) {
            int ready = counter(low_ready);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            double2 v = rd_base[half];
            int vf = rd_frame[half];
            ready = uniform(ready);
            if (__builtin_expect(ready < generation, 0)) {
                while (ready < generation && budget > 0) {
                    --budget;
                    ready = counter(low_ready);
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    v = rd_base[half];
                    vf = rd_frame[half];
                    ready = uniform(ready);
                }
                lost = lost || ready < generation;
            }
            if (lane < halo) {
                v_blank = v.x;
                v_label = v.y;
                frame = vf;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            if (lane == 0) __hip_atomic_store(my_done, generation, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    };

    // Label value of pair j-1 after the last step, in that pair's frame (0 for pair 0: the shift
    // leaves lane 0 what it had).
    int prev_lo = 0, prev_hi = 0;
    auto from_prev_pair = [&](double mine) { return shift_up(mine, prev_lo, prev_hi); };
    const unsigned long long counted = __ballot(j >= 0 && j <= L);   // the lanes with a pair of the label (the others hold zeros)
    unsigned long long rough = ~0ull;                    // lanes whose frame lies far below that of the lane below (kSmoothFrames)
    auto shift_up_int = [](int v) { return __builtin_amdgcn_update_dpp(kNoExponent, v, 0x138, 0xf, 0xf, false); };

    // New frames after a chunk.  (A pair whose window holds no mass yet gets kNoExponent: its
    // values are zero and stay zero whatever the exponent.)
    auto renew_frames = [&]() {
        const double top = fmax(v_blank, v_label);
        const int mine = (top > 0.0) ? frame + __builtin_amdgcn_frexp_exp(top) : kNoExponent;
        int window = mine;
#pragma unroll
        for (int k = 0; k < kChunk; ++k) window = window_max_step(window, mine);
        window = lane_frame(window, mine);
        const int rise = frame - window;
        v_blank = __builtin_amdgcn_ldexp(v_blank, rise);
        v_label = __builtin_amdgcn_ldexp(v_label, rise);
        frame = window;
        // 2^1023 is the largest factor there is; a pair that far below its neighbour has been
        // rounded away already.
        const int down = shift_up_int(window) - window;
        const int below = min(max(down, -1100), 1023);
        scale = __builtin_amdgcn_ldexp(1.0, below);
        skip_scale = skip_ok ? scale : 0.0;
        rough = __ballot(down > kSmoothFrames) & counted;
    };
    auto renewal_due = [&]() {
        return ((__ballot(outside_easy_range(fmax(v_blank, v_label))) & counted) | rough) != 0;
    };

    auto end_chunk = [&]() {
        bool handed = false;
        if (kSync == Sync::kHalo) {
            if (--until_hand_over == 0) {
                hand_over();                             // (the halo lanes come back with other frames)
                until_hand_over = chunks_per_hand_over;
                handed = true;
            }
        }
        // (Only chains of one wavefront put renewals off: the wavefronts of a longer chain keep in step
        // best when all of them do the same work per chunk; measured 5 % slower otherwise.)
        if (kSync != Sync::kNone || handed || renewal_due()) renew_frames();
        // the next chunk's exponent row
        xp += xstride;
        if (kMode == Mode::kGrad) lattice_store(xp, frame);
    };
    // One step.  The blank state sums its own value and the label of the pair before; the label state
    // its own value, the old blank and, where the skip is allowed, that label too:
    //   label' = fma(previous label, skip, label + blank) * emission.
    // A lone wavefront on its SIMD issues an instruction every 2 ns, but one that reads the result of
    // the instruction before it only after 4 ns, and of the one before that after 3 (measured on gfx950
    // with chains of dependent v_fma_f64).  So the statements are in the order of issue (pin keeps the
    // compiler from moving them), and none needs a result younger than two instructions: the sum and
    // the conversions fill the time the two DPP moves take, the address the time of the multiply-adds.
    auto pin = []() { __builtin_amdgcn_sched_barrier(0); };
    auto advance = [&](double eb_d, float el) {
#pragma clang fp contract(off)                           // (a product stays a product: fused into the next step's sum it would tie the steps together)
        const double prev = from_prev_pair(v_label);
        pin();
        const double u = v_blank + v_label;
        pin();
        const double el_d = static_cast<double>(el);
        pin();
        i_label = __builtin_fma(prev, skip_scale, u);
        pin();
        i_blank = __builtin_fma(prev, scale, v_blank);
        pin();
        uint32_t* const here = op;
        op += ostride;
        pin();
        v_label = i_label * el_d;
        pin();
        v_blank = i_blank * eb_d;
        pin();
        if (kMode == Mode::kGrad) lattice_store(here, static_cast<uint32_t>(__double2hiint(kBackward ? i_label : v_label)));
        pin();
    };

    // step 0
    {
        const float el = *ep;
        v_blank = i_blank * blank_of(blank_window(0), 0);
        v_label = i_label * static_cast<double>(el);
        if (kMode == Mode::kGrad) {
            lattice_store(op, static_cast<uint32_t>(__double2hiint(kBackward ? i_label : v_label)));
            lattice_store(xp, frame);                    // exponent row 0: step 0 and the first chunk
        }
        op += ostride;
    }

    // Emissions of steps 1..: two register sets, one in use, one being filled (as run_chain_log).
    // Three register sets: a chunk's emissions are requested two chunks before their use (with two sets,
    // one chunk ahead, a seventh of a single-wavefront chain's time went into waiting for them).
    float el_a[kChunk], el_b[kChunk], el_c[kChunk];
    double eb_a[kChunk] = {}, eb_b[kChunk] = {}, eb_c[kChunk] = {};
    // (Scalar loads return in any order, so a wavefront can only wait for all of them: the set in use is
    // waited for before the other set's load goes out, while that wait is still free.)
    // The label emissions of the chunk at s0 go into `el`, two chunks ahead of their use; the blank's
    // scalars into `eb`, the set of the chunk that runs next, for the chunk before s0, so that only two of
    // the three scalar sets are in use at any time (48 scalar registers for them were more than the kernel
    // has: the compiler parked a set in vector lanes and fetched it back, 32 moves per round).
    auto fetch = [&](float (&el)[kChunk], double (&eb)[kChunk], const double (&in_use)[kChunk], int s0) {
        asm volatile("" : : "s"(in_use[0]), "s"(in_use[kChunk - 1]));
        const double* const w = blank_window(blank64_chunk_with(s0));
#pragma unroll
        for (int i = 0; i < kChunk; ++i) eb[i] = blank_of(w, i);
        if (direct) {
            fetch_frames<kBackward>(ep, eadvance, el);
            return;
        }
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            ep += estride;
            el[i] = *ep;
        }
    };
    auto run = [&](const float (&el)[kChunk], const double (&eb)[kChunk], int s0, bool whole) {
        if (whole) {
#pragma unroll
            for (int i = 0; i < kChunk; ++i) advance(eb[i], el[i]);
        } else {
#pragma unroll
            for (int i = 0; i < kChunk; ++i)
                if (s0 + i < Tb) advance(eb[i], el[i]);
        }
    };
    chain_schedule3(Tb, [&](int s0) { fetch(el_a, eb_c, eb_b, s0); __builtin_amdgcn_sched_barrier(0); },
                    [&](int s0) { fetch(el_b, eb_a, eb_c, s0); __builtin_amdgcn_sched_barrier(0); },
                    [&](int s0) { fetch(el_c, eb_b, eb_a, s0); __builtin_amdgcn_sched_barrier(0); },
                    [&](int s0, bool whole) { run(el_a, eb_a, s0, whole); }, [&](int s0, bool whole) { run(el_b, eb_b, s0, whole); },
                    [&](int s0, bool whole) { run(el_c, eb_c, s0, whole); }, end_chunk);

    if (!kBackward) {
        // p = alpha_{T-1}(2L) + alpha_{T-1}(2L-1), from the lane of pair L (exact, as is the
        // lane below it: see run_chain_log).
        const double from_below = from_prev_pair(v_label) * scale;
        if (active && j == L) {
            // p = mantissa * 2^exponent, mantissa in [0.5, 1)
            const double p = v_blank + from_below;
            const double mantissa = __builtin_amdgcn_frexp_mant(p);
            const int exponent = frame + __builtin_amdgcn_frexp_exp(p);
            // (in double: once per chain, and a cost near zero, p near 1, would keep few of a float logarithm's bits)
            const double l2 = static_cast<double>(exponent) + ::log2(mantissa);
            lattice_store(&logp[u], (p > 0.0) ? pack_state(1.0 / mantissa, -exponent) : 0.0);     // 1 / p
            const float cost = (p > 0.0) ? static_cast<float>(-l2 * kLn2) : __builtin_inff();
            if (kSync == Sync::kHalo && kMode == Mode::kLoss) hl->cost = cost;
            else costs[u] = cost;
        }
    }
    if (kSync == Sync::kHalo && kMode == Mode::kLoss) {
        // as in run_chain_log: the wavefront that finishes last writes the cost
        if (lost && lane == 0) hl->gave_up = 1;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        int before = 0;
        if (lane == 0)
            before = __hip_atomic_fetch_add(&hl->finished, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        before = __builtin_amdgcn_readfirstlane(before);
        if (before == m.waves - 1 && lane == 0) {
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int any_lost = __hip_atomic_load(&hl->gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            const float cost = hl->cost;
            costs[u] = any_lost ? __uint_as_float(0x7FC00000u) : cost;
        }
    } else if (kSync == Sync::kHalo && lost && lane == 0) {
        lattice_store(&chain_err[u], 1);
    }
}

// Linear-domain chains of more than 64 pairs: a lane owns two neighbouring pairs, A = 2q and
// B = 2q + 1 (q = wave * (64 - halo) + lane), so a wavefront covers 128 pairs and most labels need
// one or two wavefronts instead of two to four.  Pair A takes the label of pair B of the lane
// below (one DPP shift and `scale`, as in run_chain_linear), pair B the label of pair A of its own
// lane: the two recursions of a lane are independent within a step and fill each other's issue
// gaps.  Both pairs share the lane's frame; mass moves up half a lane per step, so the window
// of a renewal is this lane and the kChunk / 2 lanes below it, and a halo of h lanes stays exact
// for 2h steps (hand-over every 2h steps: h is a multiple of 4).
// The two label states of a lane are neighbours in the lattice row and go out in one 16-byte
// store; where pair B has no label state (the lane of the last pair) its half falls on one of
// the row's two unused columns.
struct alignas(4) LabelStatePair { uint32_t lo, hi; };   // two neighbouring columns of a lattice row
struct alignas(4) ExponentPair { int lo, hi; };

template <bool kBackward, Mode kMode, bool kSymbolMajor>
__device__ __forceinline__ void run_chain_linear2(const Utt m, const int u, const int* __restrict__ labels,
                                                  const float* __restrict__ emit_blank,
                                                  const double* __restrict__ emit_blank64,
                                                  const float* __restrict__ emit_label,
                                                  uint32_t* __restrict__ out, int* __restrict__ out_exponents,
                                                  double* __restrict__ logp,
                                                  float* __restrict__ costs, int* __restrict__ chain_err,
                                                  uint32_t* __restrict__ sink, void* lds)
{
    static_assert(kMode == Mode::kGrad || !kBackward, "only the gradient needs the backward chain");
    static_assert(kMode != Mode::kBest, "the maximum recursion runs in the log domain");
    const int L = m.L, Tb = m.Tb;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // (uniform: in a scalar register)
    const int halo = m.halo2, waves = m.waves2;
    const int q = wave * (64 - halo) + lane;
    const int ja = 2 * q, jb = 2 * q + 1;                // the lane's pairs, in the chain's own order
    const int* lab = labels + m.lab_off;
    const bool has_a = ja < L, has_b = jb < L;           // label states (pair L has a blank state only)
    const bool active = (wave == 0 || lane >= halo) && ja <= L;
    const int lia = kBackward ? (L - 1 - ja) : ja;       // label index of pair A's label state
    const int lib = kBackward ? (lia - 1) : (lia + 1);
    const int back = kBackward ? 1 : -1;                 // label index of the pair before = index + back
    const bool skip_a = has_a && ja >= 1 && lab[lia] != lab[lia + back];
    const bool skip_b = has_b && lab[lib] != lab[lib + back];

    const int f0 = kBackward ? (Tb - 1) : 0;
    const int fdir = kBackward ? -1 : 1;
    constexpr bool direct = kSymbolMajor;                // see run_chain_log
    // A pair without a label state reads a constant probability 0 and stays there.
    const float* epa = emit_label + label_emission_offset(m, has_a, direct, has_a ? lab[lia] : 0, lia, f0, kZeroEmission);
    const float* epb = emit_label + label_emission_offset(m, has_b, direct, has_b ? lab[lib] : 0, lib, f0, kZeroEmission);
    const int advance_a = static_cast<int>(label_emission_step(m, has_a, true, fdir)) * kChunk;
    const int advance_b = static_cast<int>(label_emission_step(m, has_b, true, fdir)) * kChunk;
    const int64_t stride_a = label_emission_step(m, has_a, false, fdir);
    const int64_t stride_b = label_emission_step(m, has_b, false, fdir);
    (void)emit_blank;                                    // the blank's probability: fp64 scalars (see run_chain_linear)
    const double* const bq = emit_blank64;
    auto blank_window = [&](int s0) { return bq + blank64_window(m, f0, fdir, s0); };
    auto blank_of = [&](const double* w, int i) { return w[kBackward ? kChunk - 1 - i : i]; };
    // Output: label state i sits in column 1 + i; the lane's two are columns 1 + min(lia, lib) and
    // the next one.  (has_a false: nothing of this lane is kept.)
    const bool stores = kMode == Mode::kGrad && active && has_a;
    const int pitch = static_cast<int>(lattice_pitch(L));
    const int first_column = 1 + (kBackward ? lib : lia);
    uint32_t* op = stores ? out + m.ab_off + static_cast<int64_t>(f0) * pitch + first_column : sink;
    const int64_t ostride = stores ? static_cast<int64_t>(fdir) * pitch : 0;
    int* xp = stores ? out_exponents + m.ab_off + first_column : reinterpret_cast<int*>(sink);
    const int64_t xstride = stores ? pitch : 0;

    HaloHeader* const hl = static_cast<HaloHeader*>(lds);
    const int last_wave = waves - 1;
    int budget = m.poll_budget;
    bool lost = false;
    const int chunks_per_hand_over = 2 * halo / kChunk;
    int until_hand_over = chunks_per_hand_over;
    int generation = 0;
    const int wr_slot = (halo > 0 && lane >= 64 - halo) ? lane - (64 - halo) : 0;
    const int rd_slot = lane < halo ? lane : 0;
    Halo2Wave* const mine_lds = halo_wave<Halo2Wave>(lds, wave);
    Halo2Wave* const below_lds = halo_wave<Halo2Wave>(lds, wave > 0 ? wave - 1 : 0);
    Halo2Wave* const above_lds = halo_wave<Halo2Wave>(lds, wave < last_wave ? wave + 1 : wave);

    double ia_blank = (ja == 0) ? 1.0 : 0.0, ia_label = (ja == 0 && has_a) ? 1.0 : 0.0;
    double ib_blank = 0.0, ib_label = 0.0;
    double va_blank, va_label, vb_blank, vb_label;
    int frame = 0;
    double scale = 1.0;                                  // 2^(frame of the lane below - frame)
    double skip_a_scale = skip_a ? 1.0 : 0.0;
    const double skip_b_one = skip_b ? 1.0 : 0.0;

    auto uniform = [](int v) { return __builtin_amdgcn_readfirstlane(v); };
    auto generation_of = [&](const int2* tag) {
        return __hip_atomic_load(&tag->y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    auto read_tag = [&](const int2* tag) {
        const unsigned long long w = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(tag),
                                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        return make_int2(static_cast<int>(w), static_cast<int>(w >> 32));
    };
    auto write_tag = [&](int2* tag, int frame_of_lane, int number) {
        __hip_atomic_store(reinterpret_cast<unsigned long long*>(tag),
                           (static_cast<unsigned long long>(static_cast<unsigned>(number)) << 32) |
                               static_cast<unsigned>(frame_of_lane),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    int above_seen = 0;
    // Hand-over g: first take the halo lanes' exact state from the wavefront below, then pass the
    // top `halo` lanes up.  An entry is a lane's four values and, in a last word, its frame and
    // the number g; LDS operations of a wavefront complete in order, so a reader that finds g in
    // the last word finds the values of hand-over g in the others.  A boundary's buffer holds
    // kRing hand-overs.  Before it overwrites the one that held hand-over g - kRing, a wavefront
    // makes sure that the one above has taken that: a wavefront publishes g only after its own
    // reads of g (the last one, which has nothing to hand up, publishes a bare number), so what
    // it has published says how far it has read; that reading was requested at the previous
    // hand-over.  (With one pair per lane this form was 4 % slower than two counters and two
    // buffers; with two pairs per lane in a crowded launch it is 9 % faster.)
    auto hand_over = [&]() {
        ++generation;
        const int half = generation & (kRing - 1);
        if (wave > 0) {
            const int2* const tag = &below_lds->tag[half][rd_slot];
            const double2* const data = &below_lds->data[half][rd_slot][0];
            int2 t = read_tag(tag);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            double2 a = data[0], b = data[1];
            int ready = uniform(t.y);
            if (__builtin_expect(ready < generation, 0)) {
                while (ready < generation && budget > 0) {
                    --budget;
                    t = read_tag(tag);
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    a = data[0];
                    b = data[1];
                    ready = uniform(t.y);
                }
                lost = lost || ready < generation;
            }
            if (lane < halo) {
                va_blank = a.x;
                va_label = a.y;
                vb_blank = b.x;
                vb_label = b.y;
                frame = t.x;
            }
        }
        if (wave < last_wave) {
            int seen = uniform(above_seen);
            if (__builtin_expect(seen < generation - kRing, 0)) {
                while (seen < generation - kRing && budget > 0) {
                    --budget;
                    seen = uniform(generation_of(&above_lds->tag[half][0]));
                }
                lost = lost || seen < generation - kRing;
            }
            if (lane >= 64 - halo) {
                mine_lds->data[half][wr_slot][0] = make_double2(va_blank, va_label);
                mine_lds->data[half][wr_slot][1] = make_double2(vb_blank, vb_label);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                write_tag(&mine_lds->tag[half][wr_slot], frame, generation);
            }
            above_seen = generation_of(&above_lds->tag[(half + 1) & (kRing - 1)][0]);
        } else if (wave > 0) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            if (lane == 0) write_tag(&mine_lds->tag[half][0], 0, generation);
        }
    };

    int prev_lo = 0, prev_hi = 0;
    auto from_lane_below = [&](double mine) { return shift_up(mine, prev_lo, prev_hi); };
    auto shift_up_int = [](int v) { return __builtin_amdgcn_update_dpp(kNoExponent, v, 0x138, 0xf, 0xf, false); };

    auto renew_frames = [&]() {
        const double top = fmax(fmax(va_blank, va_label), fmax(vb_blank, vb_label));
        const int mine = (top > 0.0) ? frame + __builtin_amdgcn_frexp_exp(top) : kNoExponent;
        int window = mine;
#pragma unroll
        for (int k = 0; k < kChunk / 2; ++k) window = window_max_step(window, mine);
        window = lane_frame(window, mine);
        const int rise = frame - window;
        va_blank = __builtin_amdgcn_ldexp(va_blank, rise);
        va_label = __builtin_amdgcn_ldexp(va_label, rise);
        vb_blank = __builtin_amdgcn_ldexp(vb_blank, rise);
        vb_label = __builtin_amdgcn_ldexp(vb_label, rise);
        frame = window;
        const int down = min(max(shift_up_int(window) - window, -1100), 1023);
        scale = __builtin_amdgcn_ldexp(1.0, down);
        skip_a_scale = skip_a ? scale : 0.0;
    };

    auto store = [&](double label_a, double label_b) {
        if (kMode == Mode::kGrad) {
            const uint32_t a = static_cast<uint32_t>(__double2hiint(label_a));
            const uint32_t b = static_cast<uint32_t>(__double2hiint(label_b));
            // (one 8-byte word: b's value in the upper half when a's column comes first)
            lattice_store(reinterpret_cast<unsigned long long*>(op),
                          kBackward ? (static_cast<unsigned long long>(a) << 32) | b : (static_cast<unsigned long long>(b) << 32) | a);
        }
        op += ostride;
    };
    // both label states of the lane share its frame
    auto store_frame = [&]() {
        if (kMode == Mode::kGrad)
            lattice_store(reinterpret_cast<unsigned long long*>(xp),
                          (static_cast<unsigned long long>(static_cast<unsigned>(frame)) << 32) | static_cast<unsigned>(frame));
    };
    auto first_step = [&](double ebd, float ela, float elb) {
        va_blank = ia_blank * ebd;
        va_label = ia_label * static_cast<double>(ela);
        vb_blank = ib_blank * ebd;
        vb_label = ib_label * static_cast<double>(elb);
        store(kBackward ? ia_label : va_label, kBackward ? ib_label : vb_label);
    };
    auto end_chunk = [&]() {
        if (--until_hand_over == 0) {
            hand_over();
            until_hand_over = chunks_per_hand_over;
        }
        renew_frames();
        xp += xstride;                                   // the next chunk's exponent row
        store_frame();
    };
    // One step.  A lone wavefront on its SIMD issues an instruction every 2 ns, but one that reads the
    // result of the instruction before it only after 4 ns, and of the one before that after 3 (measured
    // on gfx950 with chains of dependent v_fma_f64).  The step is therefore written so that no
    // instruction needs a result younger than two instructions, and the order of the statements is
    // the order of issue (pin): the sums that do not need the neighbour's value come first, while the
    // two DPP moves are on their way, and the two pairs' products alternate.
    //   label' = (label + blank + skip * previous label) * emission, as fma(previous, skip, label + blank)
    auto pin = []() { __builtin_amdgcn_sched_barrier(0); };
    auto advance = [&](double eb_d, float ela, float elb) {
#pragma clang fp contract(off)                           // (a product stays a product: fusing it into the next step's sum would tie the steps together)
        const double prev = from_lane_below(vb_label);
        pin();
        const double ub = vb_blank + vb_label;
        pin();
        const double ua = va_blank + va_label;
        pin();
        ib_blank = vb_blank + va_label;
        pin();
        const double ela_d = static_cast<double>(ela);
        pin();
        ib_label = __builtin_fma(va_label, skip_b_one, ub);
        pin();
        ia_label = __builtin_fma(prev, skip_a_scale, ua);
        pin();
        ia_blank = __builtin_fma(prev, scale, va_blank);
        pin();
        const double elb_d = static_cast<double>(elb);
        pin();
        va_label = ia_label * ela_d;
        pin();
        vb_label = ib_label * elb_d;
        pin();
        va_blank = ia_blank * eb_d;
        pin();
        vb_blank = ib_blank * eb_d;
        pin();
        store(kBackward ? ia_label : va_label, kBackward ? ib_label : vb_label);
        pin();
    };

    // step 0
    store_frame();                                       // exponent row 0: step 0 and the first chunk
    first_step(blank_of(blank_window(0), 0), *epa, *epb);

    float ela_a[kChunk], elb_a[kChunk], ela_b[kChunk], elb_b[kChunk], ela_c[kChunk], elb_c[kChunk];
    double eb_a[kChunk] = {}, eb_b[kChunk] = {}, eb_c[kChunk] = {};
    // (label emissions two chunks ahead, the blank's scalars one: see run_chain_linear)
    auto fetch = [&](float (&ela)[kChunk], float (&elb)[kChunk], double (&eb)[kChunk], const double (&in_use)[kChunk], int s0) {
        asm volatile("" : : "s"(in_use[0]), "s"(in_use[kChunk - 1]));     // (see run_chain_linear)
        const double* const w = blank_window(blank64_chunk_with(s0));
#pragma unroll
        for (int i = 0; i < kChunk; ++i) eb[i] = blank_of(w, i);
        if (direct) {
            fetch_frames<kBackward>(epa, advance_a, ela);
            fetch_frames<kBackward>(epb, advance_b, elb);
            return;
        }
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            epa += stride_a;
            epb += stride_b;
            ela[i] = *epa;
            elb[i] = *epb;
        }
    };
    auto run = [&](const float (&ela)[kChunk], const float (&elb)[kChunk], const double (&eb)[kChunk], int s0, bool whole) {
        if (whole) {
#pragma unroll
            for (int i = 0; i < kChunk; ++i) advance(eb[i], ela[i], elb[i]);
        } else {
#pragma unroll
            for (int i = 0; i < kChunk; ++i)
                if (s0 + i < Tb) advance(eb[i], ela[i], elb[i]);
        }
    };
    chain_schedule3(Tb, [&](int s0) { fetch(ela_a, elb_a, eb_c, eb_b, s0); __builtin_amdgcn_sched_barrier(0); },
                    [&](int s0) { fetch(ela_b, elb_b, eb_a, eb_c, s0); __builtin_amdgcn_sched_barrier(0); },
                    [&](int s0) { fetch(ela_c, elb_c, eb_b, eb_a, s0); __builtin_amdgcn_sched_barrier(0); },
                    [&](int s0, bool whole) { run(ela_a, elb_a, eb_a, s0, whole); },
                    [&](int s0, bool whole) { run(ela_b, elb_b, eb_b, s0, whole); },
                    [&](int s0, bool whole) { run(ela_c, elb_c, eb_c, s0, whole); }, end_chunk);

    if (!kBackward) {
        // p = alpha_{T-1}(2L) + alpha_{T-1}(2L-1): the blank of pair L and the label of pair L - 1.
        // L even: pair L is this lane's A, pair L - 1 the B of the lane below; L odd: pair L is B.
        const double from_below = from_lane_below(vb_label) * scale;
        if (active && (ja == L || jb == L)) {
            const double p = (ja == L) ? va_blank + from_below : vb_blank + va_label;
            const double mantissa = __builtin_amdgcn_frexp_mant(p);         // [0.5, 1)
            const int exponent = frame + __builtin_amdgcn_frexp_exp(p);
            // (in double: once per chain, and a cost near zero, p near 1, would keep few of a float logarithm's bits)
            const double l2 = static_cast<double>(exponent) + ::log2(mantissa);
            lattice_store(&logp[u], (p > 0.0) ? pack_state(1.0 / mantissa, -exponent) : 0.0);     // 1 / p
            const float cost = (p > 0.0) ? static_cast<float>(-l2 * kLn2) : __builtin_inff();
            if (kMode == Mode::kLoss) hl->cost = cost;
            else costs[u] = cost;
        }
    }
    if (kMode == Mode::kLoss) {
        // as in run_chain_log: the wavefront that finishes last writes the cost
        if (lost && lane == 0) hl->gave_up = 1;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        int before = 0;
        if (lane == 0)
            before = __hip_atomic_fetch_add(&hl->finished, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        before = __builtin_amdgcn_readfirstlane(before);
        if (before == waves - 1 && lane == 0) {
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int any_lost = __hip_atomic_load(&hl->gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            const float cost = hl->cost;
            costs[u] = any_lost ? __uint_as_float(0x7FC00000u) : cost;
        }
    } else if (lost && lane == 0) {
        lattice_store(&chain_err[u], 1);
    }
}

// Where the chains of a launch leave their states: value and exponent blocks of both directions
// (see "lattice storage").  In the modes without a backward chain the forward value block receives
// the predecessor choices (Mode::kBest) or nothing.
struct LatticeOut {
    uint32_t* alpha;
    int* alpha_exponents;
    uint32_t* beta;
    int* beta_exponents;
};

// ---- gradient rows inside the lattice launch (kTaskRows in the launcher's header) ----------------
// What the workgroups after the chains' get besides the chains' arguments.
struct WorkerArgs {
    const void* x;            // activations and gradient tensor, of type `dtype`
    void* grads;
    const int* links;
    const float* lse;
    const int* tasks;         // the list of tasks: die[kXcds + 1], prefix[2B + 1], info[2B], first[2B]
    int* done;                // per utterance: wavefronts of its chains that have ended
    int* where;               // per chain: 1 + the die its workgroup runs on
    int* leftover;            // per utterance: set if a worker had to leave its rows to the gradient launch
    int n_tasks;              // 0: the launch has no workers
    int n_entries;
    int n_chains;
    int n_cu;
    int rounds;               // the launch has rounds x n_cu workgroups; the first n_chains of every round do not work
    int worker_waves;         // wavefronts of a working workgroup that have a piece of LDS to work in
    int T, B, A, blank, Lmax;
    int dtype;
    int lds_ints;             // ints of dynamic LDS of the launch's workgroups
    // (used by the chains as well)
    const int* row_flags;     // narrow softmax launch's words (rows_flagged), or nullptr: the records' flags say it all
    int flag_blocks;          // ... per utterance
    int* domain;              // per utterance: did its chains run in the log domain (published by the forward chain)
    int* host_flag;           // pinned host word that receives host_flag_value: the image may be reused (or nullptr)
    int host_flag_value;
    const int* status_words;  // device-resident metadata built by the narrow softmax launch: per utterance, nonzero if
    int* status_out;          // invalid; gathered into the caller's status word by this launch (or nullptr)
    int status_count;
    int skip_directions;      // bit 0: leave the forward chains out, bit 1: the backward chains (measurements only)
};

// The die (XCD) this wavefront runs on: each has an L2 of its own.
__device__ __forceinline__ int this_xcd() { return static_cast<int>(__builtin_amdgcn_s_getreg(63508) & 15u); }   // XCC_ID, 32 bits

// How a chain hands its lattice to the workers without a device-wide cache write-back (which,
// with the matching invalidation on the workers' side, was measured to lengthen the running chains
// by half): the L2 of a die is the point at which all its compute units agree, a chain's stores are
// complete once that L2 has them, and workgroups are dealt to the dies in turn, so that the workers
// of a die can be given the utterances whose chains ran there.  A chain's first wavefront publishes
// the die it finds itself on; a worker that finds itself on another die than both chains of an
// utterance does not touch it and marks the utterance for the gradient launch that follows.
__device__ __forceinline__ void chain_started(const WorkerArgs& wk, int chain)
{
    if (wk.n_tasks > 0 && threadIdx.x == 0)
        __hip_atomic_store(&wk.where[chain], this_xcd() + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// A chain's wavefront has ended.  Once all its stores have completed (the L2 has them) it counts
// itself in; the last wavefront of the chain's workgroup to do so moves the utterance's counter,
// which therefore reaches 2 when both chains have ended.
__device__ __forceinline__ void chain_ended(const WorkerArgs& wk, int u, int waves, void* lds)
{
    if (wk.n_tasks == 0 || u < 0) return;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");      // (waits for the stores; no cache operation)
    __builtin_amdgcn_s_waitcnt(0);
    bool last = true;
    if (lds) {
        int before = 0;
        if ((threadIdx.x & 63) == 0)
            before = __hip_atomic_fetch_add(&static_cast<HaloHeader*>(lds)->finished, 1, __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_WORKGROUP);
        last = __builtin_amdgcn_readfirstlane(before) == waves - 1;
    }
    if (last && (threadIdx.x & 63) == 0)
        __hip_atomic_fetch_add(&wk.done[u * kDoneStride], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}


// What a wavefront of a lattice workgroup has done: the utterance whose chain it ran to its end
// (-1: none) and the number of wavefronts of that chain.
struct ChainRun {
    int u, waves;
};

template <Sync kSync, Mode kMode, bool kSymbolMajor>
__device__ __forceinline__ ChainRun lattice_body(const Utt* __restrict__ meta, const int* __restrict__ order,
                                             const int* __restrict__ labels,
                                             const float* __restrict__ emit_blank, const double* __restrict__ emit_blank64,
                                             const float* __restrict__ emit_label,
                                             const LatticeOut lat,
                                             double* __restrict__ logp, float* __restrict__ costs,
                                             int* __restrict__ chain_err, uint32_t* __restrict__ sink,
                                             void* lds, const WorkerArgs& wk)
{
    // The first workgroup of the launch tells the host that the pinned image of the call is free
    // again (calls whose softmax launch read the image itself: this launch follows it).
    if (blockIdx.x == 0 && threadIdx.x == 0 && wk.host_flag)
        __hip_atomic_store(wk.host_flag, wk.host_flag_value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    // ... and gathers the per-utterance verdicts of a softmax launch that built the records itself.
    if (blockIdx.x == 0 && threadIdx.x < 64 && wk.status_out) {
        bool bad = false;
        for (int i = threadIdx.x; i < wk.status_count; i += 64) bad = bad || wk.status_words[i] != 0;
        const bool any = __ballot(bad) != 0;
        if (threadIdx.x == 0) *wk.status_out = any ? CTC_STATUS_INVALID_VALUE : CTC_STATUS_SUCCESS;
    }
    // Lanes with nothing to store write to a sink: 64 bytes of it per wavefront of the launch.  (One
    // address for the whole launch was what a crowded launch waited for: every store instruction of
    // every chain carried a write to it, and they all met in one channel of each die's L2.  512
    // utterances of 20 symbols and 740 frames: 59 -> 40 us.  Writing to an unused column of the
    // chain's own rows instead was slower than either in launches that are not crowded.)
    sink += (static_cast<size_t>(blockIdx.x) * kSinkWaves + (threadIdx.x >> 6)) * (kSinkBytes / sizeof(uint32_t));
    const int chain = order[blockIdx.x];           // utterance * 2 + direction
    if (chain < 0) return {-1, 0};      // device-planned batches launch a workgroup per utterance and direction, running or not
    // (measurements of the recursions one after the other: a launch that leaves one direction out)
    if (kMode == Mode::kGrad && ((wk.skip_directions >> (chain & 1)) & 1)) return {-1, 0};
    const int u = chain >> 1;
    const bool forward = kMode != Mode::kGrad || (chain & 1) == 0;
    const Utt m = meta[u];
    if (!(m.flags & kUttRuns)) return {-1, 0};     // (a run order built on the device lists every utterance)
    // Which recursion: the barrier kernel and the maximum recursion have the log domain only;
    // otherwise the flag that the softmax launch may have raised decides.  A linear-domain chain
    // gives one pair or two to a lane as the launcher planned it (two_pairs_per_lane).
    const bool in_log_domain = kSync == Sync::kBarrier || kMode == Mode::kBest || (m.flags & kUttLogDomain) != 0 ||
                               rows_flagged(wk.row_flags, u, wk.flag_blocks, m.Tb);
    // (for the gradient, which must know where each chain's exponent rows are: a word per direction)
    if (kMode == Mode::kGrad && threadIdx.x == 0) wk.domain[2 * u + (forward ? 0 : 1)] = in_log_domain ? 1 : 0;
    const bool two_pairs = kSync == Sync::kHalo && !in_log_domain && (m.flags & kUttTwoPairs) != 0;
    const int waves = two_pairs ? m.waves2 : m.waves;
    const bool idle = static_cast<int>(threadIdx.x >> 6) >= waves;
    if (kSync == Sync::kHalo) {
        // the exchange buffer in use starts with every counter and hand-over number at zero
        // (every wavefront of the workgroup clears its own block, whether it takes part or not)
        HaloHeader* hl = static_cast<HaloHeader*>(lds);
        if (two_pairs) {
            int* tags = reinterpret_cast<int*>(&halo_wave<Halo2Wave>(lds, threadIdx.x >> 6)->tag[0][0]);
            for (int i = threadIdx.x & 63; i < kRing * kHalo2Lanes * 2; i += 64) tags[i] = 0;
        } else if ((threadIdx.x & 63) == 0) {
            HaloWave* w = halo_wave<HaloWave>(lds, threadIdx.x >> 6);
            w->ready = 0;
            w->done = 0;
        }
        if (threadIdx.x == 0) {
            hl->finished = 0;
            hl->gave_up = 0;
        }
        __syncthreads();
        if (idle) return {-1, 0};
    } else if (kSync == Sync::kBarrier) {
        if (idle) {
            // Nothing to compute, but keep meeting the barriers of the working wavefronts:
            // one per recursion step, plus the forward chain's final exchange.
            const int barriers = (m.Tb - 1) + (forward ? 1 : 0);
            for (int i = 0; i < barriers; ++i) __syncthreads();
            return {-1, 0};
        }
    }
    if constexpr (kSync != Sync::kBarrier && kMode != Mode::kBest) {
        if (two_pairs) {
            if constexpr (kSync == Sync::kHalo) {
                if (forward)
                    run_chain_linear2<false, kMode, kSymbolMajor>(m, u, labels, emit_blank, emit_blank64, emit_label, lat.alpha, lat.alpha_exponents, logp, costs, chain_err, sink, lds);
                else
                    run_chain_linear2<true, Mode::kGrad, kSymbolMajor>(m, u, labels, emit_blank, emit_blank64, emit_label, lat.beta, lat.beta_exponents, logp, costs, chain_err, sink, lds);
            }
            return {u, waves};
        }
        if (!in_log_domain) {
            if (forward)
                run_chain_linear<false, kSync, kMode, kSymbolMajor>(m, u, labels, emit_blank, emit_blank64, emit_label, lat.alpha, lat.alpha_exponents, logp, costs, chain_err, sink, lds);
            else
                run_chain_linear<true, kSync, Mode::kGrad, kSymbolMajor>(m, u, labels, emit_blank, emit_blank64, emit_label, lat.beta, lat.beta_exponents, logp, costs, chain_err, sink, lds);
            return {u, waves};
        }
    }
    if (forward)
        run_chain_log<false, kSync, kMode, kSymbolMajor>(m, u, labels, emit_blank, emit_label, lat.alpha, lat.alpha_exponents, logp, costs, chain_err, sink, lds);
    else
        run_chain_log<true, kSync, Mode::kGrad, kSymbolMajor>(m, u, labels, emit_blank, emit_label, lat.beta, lat.beta_exponents, logp, costs, chain_err, sink, lds);
    return {u, waves};
}

// ---- gradient rows of narrow alphabets (shared by the gradient kernel and the lattice launch's workers) ----
constexpr int kAhead = 4;             // 64-state pieces of a row requested together

// The stored lattice of one utterance as the gradient kernels read it: the label states of frame t
// are one row of alpha values, one of beta values, and the exponent rows that the two chains wrote
// for the steps at which they reached that frame (exponent_row: alpha's step is t, beta's Tb-1-t).
struct LatticeRow {
    const uint32_t* a;
    const int* ea;
    const uint32_t* b;
    const int* eb;
};
struct LatticeRows {
    const uint32_t* a;
    const int* ea;
    const uint32_t* b;
    const int* eb;
    size_t pitch;
    int Tb;
    int log_domains;          // bit 0: the forward chain ran in the log domain, bit 1: the backward chain (chain_domains)
    __device__ __forceinline__ LatticeRow at(int t) const
    {
        const size_t values = static_cast<size_t>(t) * pitch;
        return {a + values, ea + static_cast<size_t>(exponent_row(t, (log_domains & 1) != 0)) * pitch,
                b + values, eb + static_cast<size_t>(exponent_row(Tb - 1 - t, (log_domains & 2) != 0)) * pitch};
    }
};
// The domains of an utterance's two chains as its chains published them (a word per direction:
// either chain may have gone over to the log domain on its own, see lattice_body).
template <bool kCoherent>
__device__ __forceinline__ int chain_domains(const int* __restrict__ domain, int b)
{
    return (lattice_load<kCoherent>(&domain[2 * b]) != 0 ? 1 : 0) | (lattice_load<kCoherent>(&domain[2 * b + 1]) != 0 ? 2 : 0);
}

// The rows t_first, t_first + t_step, ... (below tend) of utterance b, by one wavefront: lane k is
// symbol k (alphabets of at most 64 symbols).  s_slot, s_start, s_count: the grouping of the label's
// positions as ctc_gradient_narrow_kernel describes it, in LDS; g_slot: L + 1 floats of LDS of this
// wavefront's own.
// `stage` is called once, after the first row's values have been requested and before anything is read
// out of s_slot, s_start and s_count: a caller that still has to fill them does it there, so that its
// loads and the first row's are under way together.
template <typename T, bool kStreaming, bool kCoherent, typename Stage>
__device__ __forceinline__ void narrow_gradient_rows(const T* __restrict__ x, T* __restrict__ grads, const Utt m,
                                                     const int b, const LatticeOut lat,
                                                     const float* __restrict__ lse, const double* __restrict__ logp,
                                                     const int log_domains,   // decides where a row's exponents are (LatticeRows)
                                                     const int Tt, const int B, const int A, const int blank,
                                                     const int t_first, const int t_step, const int tend,
                                                     const int* s_slot, const int* s_start, const int* s_count,
                                                     float* g_slot, Stage&& stage)
{
    const int lane = threadIdx.x & 63;
    const bool runs = (m.flags & kUttRuns) != 0;
    const int L = m.L;
    const size_t pitch = static_cast<size_t>(lattice_pitch(L));
    const double packed_inverse_p = runs ? lattice_load<kCoherent>(&logp[b]) : 0.0;
    const float inverse_p = static_cast<float>(packed_inverse_p);
    const int inverse_p_exponent = __double2loint(packed_inverse_p);
    const LatticeRows rows_of{lat.alpha + m.ab_off + 1, lat.alpha_exponents + m.ab_off + 1,     // label state i sits
                              lat.beta + m.ab_off + 1, lat.beta_exponents + m.ab_off + 1,       // in column 1 + i
                              pitch, m.Tb, log_domains};
    // What a row needs from memory: the lattice words of its first kAhead * 64 label states
    // (longer labels read the rest in line), its log-sum-exp and its activations.  A row's
    // values are requested while the row before it is still being summed up out of LDS: by then
    // the registers are free again (the shares are in LDS), so the overlap costs none.
    struct RowData {
        uint32_t a[kAhead], b[kAhead];
        int ea[kAhead], eb[kAhead];
        float l2, x0;
    };
    // Row addresses are kept as running pointers of this wavefront's rows (t_first, t_first + t_step,
    // ...): the product (t x B + b) x A is formed once, not per row.
    const float* next_lse = lse + static_cast<size_t>(b) * Tt + t_first;
    const size_t row_step = static_cast<size_t>(t_step) * B * A;
    const T* next_x = x + (static_cast<size_t>(t_first) * B + b) * A;
    T* grow = grads + (static_cast<size_t>(t_first) * B + b) * A;                     // of the row being written
    // A lattice larger than the caches is read once and never again: such launches read the values
    // with loads that leave no copy behind (kStreaming), which keeps the caches for the rest (the
    // exponent rows among it: eight frames share one).
    auto value_word = [&](const uint32_t* p) {
        return kCoherent ? lattice_load<true>(p) : (kStreaming ? __builtin_nontemporal_load(p) : *p);
    };
    auto exponent_word = [&](const int* p) { return lattice_load<kCoherent>(p); };
    auto request = [&](int t, RowData& d) {
        const LatticeRow row = rows_of.at(t);
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            if (u * 64 >= L) break;                      // (the same for every lane)
            const int j = u * 64 + lane;
            if (j < L) {
                d.a[u] = value_word(row.a + j);
                d.b[u] = value_word(row.b + j);
                d.ea[u] = exponent_word(row.ea + j);
                d.eb[u] = exponent_word(row.eb + j);
            }
        }
        d.l2 = *next_lse;
        d.x0 = (lane < A) ? load_elem(next_x, lane) : 0.0f;
    };
    auto advance_request = [&]() {
        next_lse += t_step;
        next_x += row_step;
    };
    RowData cur = {};
    if (runs && t_first < tend && t_first < m.Tb) request(t_first, cur);
    stage();
    for (int t = t_first; t < tend; t += t_step, grow += row_step) {
        if (t >= m.Tb || !runs) {
            if (lane < A) store_elem(grow, lane, 0.0f);
            continue;
        }
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            if (u * 64 >= L) break;                      // (the same for every lane)
            const int j = u * 64 + lane;
            if (j < L) g_slot[s_slot[j]] = mass_share(cur.a[u], cur.ea[u], cur.b[u], cur.eb[u], inverse_p, inverse_p_exponent);
        }
        if (L > kAhead * 64) {
            const LatticeRow row = rows_of.at(t);         // this row's states past the first kAhead * 64
            for (int j = kAhead * 64 + lane; j < L; j += 64)
                g_slot[s_slot[j]] = mass_share(value_word(row.a + j), exponent_word(row.ea + j), value_word(row.b + j), exponent_word(row.eb + j),
                                               inverse_p, inverse_p_exponent);
        }
        const float l2 = cur.l2, x0 = cur.x0;
        advance_request();
        if (t + t_step < tend && t + t_step < m.Tb) request(t + t_step, cur);
        // LDS operations of one wavefront complete in program order; the fences only keep the
        // compiler from moving them across.
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        // The shares now sit in slot order, the positions of a symbol next to each other: turn
        // them into running sums (64 slots at a time, the total so far carried along), so that
        // a symbol's occupancy is the difference of two entries and the blank's 1 minus the last.
        float carried = 0.0f;
        for (int base = 0; base < L; base += 64) {
            const int slot = base + lane;
            const float sum = wave_running_sum(slot < L ? g_slot[slot] : 0.0f) + carried;
            if (slot < L) g_slot[slot] = sum;
            carried = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(sum), 63));
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (lane < A) {
            const int first = s_start[lane], count = s_count[lane];
            float o = 0.0f;
            if (count > 0) o = g_slot[first + count - 1] - (first > 0 ? g_slot[first - 1] : 0.0f);
            if (lane == blank) o = 1.0f - carried;       // the blank states share what is left of 1
            store_elem(grow, lane, fast_exp2(fmaf(x0, kLog2e, -l2)) - o);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
}

// A workgroup after the chains'.  Its wavefronts work on their own: the tasks are dealt out in
// turn over all working wavefronts of the launch (wavefront w takes tasks w, w + W, w + 2W, ...:
// no shared counter, whose traffic was measured to slow the chains severalfold), so that the
// tasks of the utterances that end last are spread over all of them.  For each task a wavefront
// waits if the utterance still has chains running, stages the grouping of the utterance's label
// in its own piece of LDS and writes the task's rows.  `lds` holds lds_ints ints: the list's table
// for the workgroup, then a piece per wavefront.
template <typename T>
__device__ __forceinline__ void gradient_worker(const WorkerArgs wk, const Utt* __restrict__ meta,
                                                const int* __restrict__ labels, const LatticeOut lat,
                                                const double* __restrict__ logp, const int* __restrict__ chain_err,
                                                float* __restrict__ costs, int* lds, const int lds_ints)
{
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int E = wk.n_entries >= 0 ? wk.n_entries : min(max(wk.tasks[kXcds], 0), 2 * wk.B), Lmax = wk.Lmax;
    int* const s_die = lds;                       // [kXcds + 1]
    int* const s_prefix = s_die + kXcds + 1;      // [E + 1]
    int* const s_info = s_prefix + E + 1;         // [E]
    int* const s_first = s_info + E;              // [E]
    const int* const prefix_in = wk.tasks + kXcds + 1;
    const int* const info_in = prefix_in + 2 * wk.B + 1;
    const int* const first_in = info_in + 2 * wk.B;
    for (int i = threadIdx.x; i <= kXcds; i += blockDim.x) s_die[i] = wk.tasks[i];
    for (int i = threadIdx.x; i <= E; i += blockDim.x) s_prefix[i] = prefix_in[i];
    for (int i = threadIdx.x; i < E; i += blockDim.x) {
        s_info[i] = info_in[i];
        s_first[i] = first_in[i];
    }
    __syncthreads();                              // the only barrier, before any wavefront waits for anything
    const int table = kXcds + 1 + 3 * E + 1, piece = 2 * Lmax + 129;
    if (wave >= wk.worker_waves || table + (wave + 1) * piece > lds_ints) return;
    int* const s_slot = lds + table + wave * piece;   // [Lmax]  as in ctc_gradient_narrow_kernel
    int* const s_start = s_slot + Lmax;               // [64]
    int* const s_count = s_start + 64;                // [64]
    float* const g_slot = reinterpret_cast<float*>(s_count + 64);   // [Lmax + 1]
    const T* const x = static_cast<const T*>(wk.x);
    T* const grads = static_cast<T*>(wk.grads);

    // This workgroup's die as the dispatcher deals them out (workgroup i to die i mod kXcds; n_cu is a
    // multiple of kXcds), its rank among the working workgroups of that die, and their number: of the
    // places n_chains .. n_cu - 1 of a round, those congruent to the die.
    const int round = static_cast<int>(blockIdx.x) / wk.n_cu, place = static_cast<int>(blockIdx.x) % wk.n_cu;
    const int die = place % kXcds;
    const int first_place = wk.n_chains + (die - wk.n_chains % kXcds + kXcds) % kXcds;
    const int per_round = (wk.n_cu - first_place + kXcds - 1) / kXcds;
    const int group = round * per_round + (place - first_place) / kXcds;
    const int stride = wk.rounds * per_round * wk.worker_waves;
    // the die's section of the list
    const int e_first = s_die[die], e_end = s_die[die + 1];
    const int ticket_first = s_prefix[e_first], ticket_end = s_prefix[e_end];
    const int xcd = this_xcd();
    int ready = -1;                               // the utterance whose chains this wavefront last found ended, here
    int staged = -1;                              // the utterance whose label grouping sits in this wavefront's LDS
    for (int ticket = ticket_first + wave * wk.rounds * per_round + group; ticket < ticket_end; ticket += stride) {
        // the run of tasks the ticket falls into
        int e = e_first;
        for (int i0 = e_first; i0 < e_end; i0 += 64) {
            const int i = i0 + lane;
            e += __popcll(__ballot(i < e_end && s_prefix[i + 1] <= ticket));
        }
        const int info = s_info[e];
        const int b = info & 0xFFFF, rows_log2 = (info >> kTaskRowsShift) & 15;
        const int t0 = (s_first[e] + ticket - s_prefix[e]) << rows_log2;
        const int tend = min(t0 + (1 << rows_log2), wk.T);
        const Utt m = meta[b];
        const bool runs = (m.flags & kUttRuns) != 0;
        if (runs && t0 < m.Tb) {
            if ((info & kTaskWaits) && b != ready) {
                // Which die do the utterance's chains run on?  They publish it as they start, at most
                // microseconds after this wavefront did.  Only if it is this die can the counter and the
                // lattice be read here (the L2 they sit in is this die's); otherwise, or if the answer
                // does not come (another die's store need not become visible here), the utterance is
                // left to the gradient launch.
                auto published = [&]() {
                    int here = 0;
                    if (lane == 0) {
                        const int f = __hip_atomic_load(&wk.where[2 * b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        const int r = __hip_atomic_load(&wk.where[2 * b + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        here = (f == 0 || r == 0) ? 0 : ((f == xcd + 1 && r == xcd + 1) ? 1 : 2);
                    }
                    return __builtin_amdgcn_readfirstlane(here);
                };
                int here = published();
                for (int polls = kWherePolls; here == 0 && polls > 0; --polls) {
                    __builtin_amdgcn_s_sleep(24);
                    here = published();
                }
                if (here != 1) {
                    if (lane == 0) wk.leftover[b] = 1;
                    continue;
                }
                const int expected = 2;          // both chains of the utterance (chain_ended)
                // (one lane asks; a sleep of some hundred nanoseconds between two questions)
                int budget = kWorkerPollBudget;
                auto ended_now = [&]() {
                    int v = 0;
                    if (lane == 0) v = __hip_atomic_load(&wk.done[b * kDoneStride], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    return __builtin_amdgcn_readfirstlane(v);
                };
                int ended = ended_now();
                while (ended < expected && budget > 0) {
                    __builtin_amdgcn_s_sleep(24);
                    --budget;
                    ended = ended_now();
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");    // (orders the loads below after the counter's)
                if (ended < expected) {
                    // (chains that never end: nothing of this task can be computed)
                    if (lane == 0) costs[b] = __uint_as_float(0x7FC00000u);
                    continue;
                }
                ready = b;
            }
            if (t0 == 0 && lane == 0 && lattice_load<true>(&chain_err[b]) != 0)
                costs[b] = __uint_as_float(0x7FC00000u);
            // the grouping of the label's positions, for this wavefront
            if (b != staged) {
            staged = b;
            s_start[lane] = 0;
            s_count[lane] = 0;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            for (int j = lane; j < m.L; j += 64) {
                const int link = wk.links[m.lab_off + j];
                s_slot[j] = link & kLinkSlotMask;
                if (link < 0) {
                    const int c = labels[m.lab_off + j];
                    s_start[c] = link & kLinkSlotMask;
                    s_count[c] = (link >> kLinkCountShift) & kLinkSlotMask;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            }
        }
        const int log_domains = (runs && t0 < m.Tb) ? chain_domains<true>(wk.domain, b) : 0;
        narrow_gradient_rows<T, false, true>(x, grads, m, b, lat, wk.lse, logp, log_domains, wk.T, wk.B, wk.A, wk.blank, t0, 1,
                                       tend, s_slot, s_start, s_count, g_slot, [] {});
    }
}

// Workgroups beyond the chains' are workers -- unless they would share a compute unit with a chain:
// the dispatcher hands workgroup i to compute unit i mod n_cu (see order_chains), a chain's
// wavefront needs its SIMD to itself, so the workgroups that would land there leave at once.
__device__ __forceinline__ bool is_worker(const WorkerArgs& wk)
{
    return wk.n_tasks > 0 && static_cast<int>(blockIdx.x) >= wk.n_chains;
}
__device__ __forceinline__ void run_worker(const WorkerArgs& wk, const Utt* __restrict__ meta,
                                           const int* __restrict__ labels, const LatticeOut lat,
                                           const double* __restrict__ logp, const int* __restrict__ chain_err,
                                           float* __restrict__ costs, int* lds)
{
    if (static_cast<int>(blockIdx.x % static_cast<unsigned>(wk.n_cu)) < wk.n_chains) return;
    if (wk.dtype == CTC_DTYPE_F32)
        gradient_worker<float>(wk, meta, labels, lat, logp, chain_err, costs, lds, wk.lds_ints);
    else
        gradient_worker<bf16_t>(wk, meta, labels, lat, logp, chain_err, costs, lds, wk.lds_ints);
}

// grid = one workgroup per entry of `order` (utterance * 2 + direction: 0 forward, 1 backward; only
// Mode::kGrad has backward chains; in the other modes `alpha` is the block that receives the
// predecessor choices, or unused).
// blockDim.x = 64 * (most wavefronts any utterance of the batch uses).
// Variant for batches whose labels all fit one wavefront: no exchange at all.
template <Mode kMode, bool kSymbolMajor>
__global__ __launch_bounds__(64)
void ctc_lattice_kernel_w1(const Utt* __restrict__ meta, const int* __restrict__ order,
                           const int* __restrict__ labels, const float* __restrict__ emit_blank,
                           const double* __restrict__ emit_blank64,
                           const float* __restrict__ emit_label,
                           const LatticeOut lat,
                           double* __restrict__ logp, float* __restrict__ costs,
                           int* __restrict__ chain_err, uint32_t* __restrict__ sink, const WorkerArgs wk)
{
    if constexpr (kMode == Mode::kGrad && kSymbolMajor) {
        if (is_worker(wk)) {
            extern __shared__ int worker_lds[];
            run_worker(wk, meta, labels, lat, logp, chain_err, costs, worker_lds);
            return;
        }
    }
    if constexpr (kMode == Mode::kGrad && kSymbolMajor) chain_started(wk, order[blockIdx.x]);
    const ChainRun ran = lattice_body<Sync::kNone, kMode, kSymbolMajor>(meta, order, labels, emit_blank, emit_blank64, emit_label, lat,
                                                                   logp, costs, chain_err, sink, nullptr, wk);
    if constexpr (kMode == Mode::kGrad && kSymbolMajor) chain_ended(wk, ran.u, ran.waves, nullptr);
}

// Multi-wavefront chains with the halo exchange.
template <Mode kMode, bool kSymbolMajor>
__global__ __launch_bounds__(1024)
void ctc_lattice_kernel(const Utt* __restrict__ meta, const int* __restrict__ order,
                        const int* __restrict__ labels, const float* __restrict__ emit_blank,
                        const double* __restrict__ emit_blank64,
                        const float* __restrict__ emit_label,
                        const LatticeOut lat,
                        double* __restrict__ logp, float* __restrict__ costs,
                        int* __restrict__ chain_err, uint32_t* __restrict__ sink, const WorkerArgs wk)
{
    extern __shared__ double2 halo_lds[];                    // halo_lds_bytes(wavefronts of the workgroup)
    if constexpr (kMode == Mode::kGrad && kSymbolMajor) {
        if (is_worker(wk)) {
            run_worker(wk, meta, labels, lat, logp, chain_err, costs, reinterpret_cast<int*>(halo_lds));
            return;
        }
    }
    if constexpr (kMode == Mode::kGrad && kSymbolMajor) chain_started(wk, order[blockIdx.x]);
    const ChainRun ran = lattice_body<Sync::kHalo, kMode, kSymbolMajor>(meta, order, labels, emit_blank, emit_blank64, emit_label, lat,
                                                                   logp, costs, chain_err, sink, halo_lds, wk);
    if constexpr (kMode == Mode::kGrad && kSymbolMajor) chain_ended(wk, ran.u, ran.waves, halo_lds);
}

// Labels too long to leave room for a halo (more than 16 * 63 pairs): 64 pairs per wavefront
// and one barrier per step.
template <Mode kMode, bool kSymbolMajor>
__global__ __launch_bounds__(1024)
void ctc_lattice_kernel_barrier(const Utt* __restrict__ meta, const int* __restrict__ order,
                                const int* __restrict__ labels, const float* __restrict__ emit_blank,
                                const double* __restrict__ emit_blank64,
                                const float* __restrict__ emit_label,
                                const LatticeOut lat,
                                double* __restrict__ logp, float* __restrict__ costs,
                                int* __restrict__ chain_err, uint32_t* __restrict__ sink, const WorkerArgs wk)
{
    __shared__ double xch[2][16];
    lattice_body<Sync::kBarrier, kMode, kSymbolMajor>(meta, order, labels, emit_blank, emit_blank64, emit_label, lat, logp,
                                               costs, chain_err, sink, &xch[0][0], wk);
}

// ---- after a forward-only chain -------------------------------------------------------------
// Most probable alignment: walk the stored predecessor choices back from the better end state.
// One wavefront per utterance; alignment is [B][T] (utterance-major): the lattice state of each
// frame (index into the blank-interleaved label), -1 for frames past the utterance's end and
// for utterances without an alignment.
//
// The walk is serial, one dependent look-up per frame, so it is kept on the scalar unit: the
// choices are fetched in tiles of kTile frames x kTile pairs, lane = pair column, one register
// per frame.  Going back kTile frames the walk moves down by at most kTile - 1 pairs (one per
// frame), so the tile whose top right corner is the walk's position holds everything those
// frames can touch.  A step is then a v_readlane at the walk's column, a shift, a mask and a
// subtraction in scalar registers, and a v_writelane that files the state for the tile's
// one coalesced store.
constexpr int kTile = 64;

__global__ __launch_bounds__(64)
void ctc_backtrace_kernel(const Utt* __restrict__ meta, const unsigned char* __restrict__ choices,
                          const double* __restrict__ end_state, const int* __restrict__ chain_err,
                          float* __restrict__ costs, int* __restrict__ alignment, int Tt)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    const Utt m = meta[b];
    int* arow = alignment + static_cast<size_t>(b) * Tt;
    const bool runs = (m.flags & kUttRuns) != 0;
    const bool bad = runs && chain_err[b] != 0;
    if (bad && lane == 0) costs[b] = __uint_as_float(0x7FC00000u);
    const int valid = (runs && !bad) ? m.Tb : 0;
    for (int t = valid + lane; t < Tt; t += 64) arow[t] = -1;
    if (valid == 0) return;

    const int P = m.L + 1;
    const unsigned char* base = choices + m.ab_off;
    // state of frame t; clamped so that no stored value can lead the reads astray
    int state = __builtin_amdgcn_readfirstlane(min(max(static_cast<int>(end_state[b]), 0), 2 * m.L));
    int t = m.Tb - 1;
    if (lane == 0) arow[t] = state;
    // Frames t, t-1, ..., 1 each hold the choice that leads to the state of the frame before.
    while (t >= 1) {
        const int pair_hi = state >> 1;                   // both states of a pair share its byte
        const int pair_lo = max(pair_hi - (kTile - 1), 0);
        const int rows = min(kTile, t);                   // frames t, t-1, ..., t-rows+1
        const unsigned col = static_cast<unsigned>(min(pair_lo + lane, pair_hi));
        // A last, partial tile repeats frame 1 in the rows below it and walks on through them:
        // those steps stay inside the tile (the state is kept >= 0) and their results are not
        // stored.  (An utterance's block is smaller than 2^31 bytes: 32-bit offsets.)
        int tile[kTile];
#pragma unroll
        for (int r = 0; r < kTile; ++r)
            tile[r] = base[static_cast<unsigned>(max(t - r, 1)) * static_cast<unsigned>(P) + col];
        int filed = 0;
#pragma unroll
        for (int r = 0; r < kTile; ++r) {
            const int c = __builtin_amdgcn_readlane(tile[r], (state >> 1) - pair_lo);
            // how far down the state of this frame came from: bits 2..3 if it is a label state
            // (odd), bits 0..1 if it is a blank
            state = max(state - ((c >> ((state << 1) & 2)) & 3), 0);
            // lane r of `filed` = state of frame t - r - 1
            asm volatile("v_writelane_b32 %0, %1, %2" : "+v"(filed) : "s"(state), "n"(r));
        }
        if (lane < rows) arow[t - 1 - lane] = filed;
        if (rows < kTile) break;
        t -= kTile;
    }
}

// ---- gradient ------------------------------------------------------------------------------
//   gamma_t(s) = alpha_t(s) * beta_t(s) / p                 mass share of state s (mass_share)
//   grad[k]    = y_t(k) - sum_{s: symbol(s) = k} gamma_t(s)
// Only the label states' gamma are computed from the stored lattice; the blank column gets
// 1 - (sum over label states), which is the blank states' share because the shares of all
// states of a frame add up to 1.  Every row of the gradient therefore sums to zero.
//
// A workgroup takes rows_per_group consecutive frames of one utterance (8 or 16 dense, 4 sparse),
// one wavefront per row at a time.  Labels and their grouping words sit in LDS; per wavefront,
// the label states' mass shares in slot order (P floats).  Everything within a row stays inside
// one wavefront, so no barrier is needed after the staging.  The first occurrence of a symbol
// adds up the run of slots of its symbol and is the only writer of that symbol's occupancy; the
// blank's L+1 states are a wavefront reduction.
//   dense  (A <= 2048): occupancies go to A floats of LDS per wavefront, then the whole row
//          y - occupancy is written, and padding rows are zero-filled;
//   sparse (wider):     the dense part of the row was written by the softmax launch; only the
//          label columns and the blank column are rewritten (no A-bin histogram).
// Dynamic LDS: 2 * L_max ints + 4 * (L_max + 1 + (dense ? A : 0)) floats.

template <typename T, bool kSparse>
__global__ __launch_bounds__(kRowThreads)
void ctc_gradient_rows_kernel(const T* __restrict__ x, T* __restrict__ grads,
                              const Utt* __restrict__ meta, const int* __restrict__ labels,
                              const int* __restrict__ links, const float* __restrict__ lse,
                              const LatticeOut lat,
                              const double* __restrict__ logp, const int* __restrict__ chain_err,
                              float* __restrict__ costs, int Tt, int B, int A, int blank, int Lmax,
                              int rows_per_group, const float* __restrict__ emit_blank,
                              const float* __restrict__ emit_label, const int* __restrict__ domain)
{
    extern __shared__ int g_lds[];
    int* s_lab = g_lds;
    int* s_lnk = g_lds + Lmax;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float* g_label = reinterpret_cast<float*>(g_lds + 2 * Lmax) + wave * (Lmax + 1 + (kSparse ? 0 : A));
    float* occ = g_label + Lmax + 1;
    const int b = blockIdx.y, t0 = blockIdx.x * rows_per_group;
    const Utt m = meta[b];
    if (t0 == 0 && tid == 0 && chain_err[b] != 0) costs[b] = __uint_as_float(0x7FC00000u);
    const bool runs = (m.flags & kUttRuns) != 0;
    const int L = m.L;
    if (runs && t0 < m.Tb) {
        for (int j = tid; j < L; j += kRowThreads) {
            s_lab[j] = labels[m.lab_off + j];
            s_lnk[j] = links[m.lab_off + j];
        }
        __syncthreads();
    }
    const size_t pitch = static_cast<size_t>(lattice_pitch(L));
    const double packed_inverse_p = runs ? logp[b] : 0.0;
    const float inverse_p = static_cast<float>(packed_inverse_p);
    const int inverse_p_exponent = __double2loint(packed_inverse_p);
    const int tend = min(t0 + rows_per_group, Tt);
    const int log_domains = runs ? chain_domains<false>(domain, b) : 0;     // decides where a row's exponents are (LatticeRows)
    const LatticeRows rows_of{lat.alpha + m.ab_off + 1, lat.alpha_exponents + m.ab_off + 1,     // label state i sits
                              lat.beta + m.ab_off + 1, lat.beta_exponents + m.ab_off + 1,       // in column 1 + i
                              pitch, m.Tb, log_domains};

    // What a row needs from memory, requested in one go before any of it is used, so that a
    // row costs one memory latency: the lattice values of the first kAhead * 64 label states
    // (longer labels read the rest in line), the row's log-sum-exp and, dense form, the first
    // 64 activations.  (Requesting the next row during the current one was measured slower:
    // the extra registers cost more wavefronts per SIMD than the overlap gains.)
    struct RowData {
        uint32_t a[kAhead], b[kAhead];
        int ea[kAhead], eb_[kAhead];
        float l2, x0;
        float e[kAhead], eb;              // sparse form: emissions of the label positions and of blank
    };
    auto request = [&](int t, RowData& d) {
        if (t >= tend || t >= m.Tb || !runs) return;
        const LatticeRow row = rows_of.at(t);
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int j = u * 64 + lane;
            if (j < L) {
                d.a[u] = row.a[j];
                d.b[u] = row.b[j];
                d.ea[u] = row.ea[j];
                d.eb_[u] = row.eb[j];
            }
        }
        d.l2 = lse[static_cast<size_t>(b) * Tt + t];
        if (!kSparse && lane < A) d.x0 = load_elem(x + (static_cast<size_t>(t) * B + b) * A, lane);
        if (kSparse) {
            const float* er = emit_label + kLabelSlack + m.e_off + static_cast<size_t>(t) * m.e_pitch;
#pragma unroll
            for (int u = 0; u < kAhead; ++u) {
                const int j = u * 64 + lane;
                if (j < L) d.e[u] = er[j];
            }
            d.eb = emit_blank[kBlankSlack + m.f_off + t];
        }
    };

    for (int t = t0 + wave; t < tend; t += 4) {
        RowData cur = {};
        request(t, cur);
        const size_t row_off = (static_cast<size_t>(t) * B + b) * A;
        T* grow = grads + row_off;
        if (t >= m.Tb || !runs) {
            if (!kSparse)
                for (int k = lane; k < A; k += 64) store_elem(grow, k, 0.0f);
            continue;
        }
        const T* xrow = x + row_off;
        const float* erow = emit_label + kLabelSlack + m.e_off + static_cast<size_t>(t) * m.e_pitch;   // sparse form only
        // Mass share of every label state; the blank states share what is left of 1.
        float zl = 0.0f;
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int j = u * 64 + lane;
            if (j < L) {
                const float gl = mass_share(cur.a[u], cur.ea[u], cur.b[u], cur.eb_[u], inverse_p, inverse_p_exponent);
                g_label[s_lnk[j] & kLinkSlotMask] = gl;
                zl += gl;
            }
        }
        if (L > kAhead * 64) {
            const LatticeRow row = rows_of.at(t);
            for (int j0 = kAhead * 64; j0 < L; j0 += kAhead * 64) {
                uint32_t a[kAhead], bb[kAhead];
                int ea[kAhead], eb[kAhead];
#pragma unroll
                for (int u = 0; u < kAhead; ++u) {
                    const int j = j0 + u * 64 + lane;
                    if (j < L) {
                        a[u] = row.a[j];
                        bb[u] = row.b[j];
                        ea[u] = row.ea[j];
                        eb[u] = row.eb[j];
                    }
                }
#pragma unroll
                for (int u = 0; u < kAhead; ++u) {
                    const int j = j0 + u * 64 + lane;
                    if (j < L) {
                        const float gl = mass_share(a[u], ea[u], bb[u], eb[u], inverse_p, inverse_p_exponent);
                        g_label[s_lnk[j] & kLinkSlotMask] = gl;
                        zl += gl;
                    }
                }
            }
        }
        const float zb = 1.0f - wave_sum(zl);
        const float l2 = cur.l2;
        if (!kSparse)
            for (int k = lane; k < A; k += 64) occ[k] = 0.0f;
        // LDS operations of one wavefront complete in program order; the fence only keeps the
        // compiler from moving them across.
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        for (int j = lane; j < L; j += 64) {
            const int link = s_lnk[j];
            if (link < 0) {                   // first occurrence of its symbol: add up its run
                const int first = link & kLinkSlotMask;
                const int count = (link >> kLinkCountShift) & kLinkSlotMask;
                float o = 0.0f;
                // Eight independent reads at a time; slots past the run add an exact zero, so
                // the order of summation is the run's own.
                for (int i0 = 0; i0 < count; i0 += 8) {
                    float g[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) g[i] = g_label[min(first + i0 + i, L - 1)];
#pragma unroll
                    for (int i = 0; i < 8; ++i) o += (i0 + i < count) ? g[i] : 0.0f;
                }
                const int c = s_lab[j];
                if (kSparse) {
                    // y of a label's symbol is its emission, which the softmax launch gathered
                    // next to its neighbours': no scattered read of the activations.
                    const int u = j >> 6;
                    float e = 0.0f;
#pragma unroll
                    for (int k = 0; k < kAhead; ++k) e = (u == k) ? cur.e[k] : e;
                    if (u >= kAhead) e = erow[j];
                    store_elem(grow, c, emission_probability(e) - o);
                } else {
                    occ[c] = o;
                }
            }
        }
        if (kSparse) {
            if (lane == 0) store_elem(grow, blank, emission_probability(cur.eb) - zb);
        } else {
            if (lane == 0) occ[blank] = zb;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            if (lane < A) store_elem(grow, lane, fast_exp2(fmaf(cur.x0, kLog2e, -l2)) - occ[lane]);
            for (int k0 = 64 + lane; k0 < A; k0 += 8 * 64) {      // eight reads in flight
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int k = k0 + u * 64;
                    v[u] = (k < A) ? load_elem(xrow, k) : 0.0f;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int k = k0 + u * 64;
                    if (k < A) store_elem(grow, k, fast_exp2(fmaf(v[u], kLog2e, -l2)) - occ[k]);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
}

// Alphabets of at most 64 symbols (the English one has 29): lane k of a row's wavefront is
// symbol k.  The shares, which sit in slot order (the positions of a symbol next to each other),
// are turned into running sums with wavefront scans; a symbol's occupancy is then the
// difference of the entries at the two ends of its run (start and length per symbol are put
// into LDS once per workgroup), the blank's is 1 minus the total, and lane k writes
// grad[k] = y_k - occupancy_k straight away: no loop over a run, no scan over the label for first
// occurrences, no occupancy array per row.  The order of the additions is fixed, so results
// repeat bitwise.
template <typename T, bool kStreaming>
__global__ __launch_bounds__(kRowThreads)
void ctc_gradient_narrow_kernel(const T* __restrict__ x, T* __restrict__ grads,
                                const Utt* __restrict__ meta, const int* __restrict__ labels,
                                const int* __restrict__ links, const float* __restrict__ lse,
                                const LatticeOut lat,
                                const double* __restrict__ logp, const int* __restrict__ chain_err,
                                float* __restrict__ costs, int Tt, int B, int A, int blank, int Lmax,
                                int rows_per_group, const int* __restrict__ only_marked,
                                const int* __restrict__ domain)
{
    // (what the rows need of the utterance is asked for in one go: each of these is a trip to memory)
    const Utt m = meta[blockIdx.y];
    const int log_domains = chain_domains<false>(domain, blockIdx.y);
    const int chain_gave_up = chain_err[blockIdx.y];
    // After a lattice launch whose workers have written the gradient: only the utterances they left.
    if (only_marked && only_marked[blockIdx.y] == 0) return;
    extern __shared__ int g_lds[];
    int* s_slot = g_lds;                         // [Lmax]  slot of each label position
    int* s_start = g_lds + Lmax;                 // [64]    first slot of each symbol's run
    int* s_count = s_start + 64;                 // [64]    length of the run (0: symbol not in the label)
    const int tid = threadIdx.x, wave = tid >> 6;
    float* g_slot = reinterpret_cast<float*>(s_count + 64) + wave * (Lmax + 1);   // mass shares in slot order
    const int b = blockIdx.y, t0 = blockIdx.x * rows_per_group;
    if (t0 == 0 && tid == 0 && chain_gave_up != 0) costs[b] = __uint_as_float(0x7FC00000u);
    const bool runs = (m.flags & kUttRuns) != 0;
    const int L = m.L;
    // The grouping of the label's positions, staged while the first rows' lattice values are on their way.
    auto stage = [&]() {
        if (!(runs && t0 < m.Tb)) return;               // (the same for the whole workgroup)
        if (tid < 64) {
            s_start[tid] = 0;
            s_count[tid] = 0;
        }
        __syncthreads();
        for (int j = tid; j < L; j += kRowThreads) {
            const int link = links[m.lab_off + j];
            const int c = labels[m.lab_off + j];         // (asked for with the link, not after it)
            s_slot[j] = link & kLinkSlotMask;
            if (link < 0) {
                s_start[c] = link & kLinkSlotMask;
                s_count[c] = (link >> kLinkCountShift) & kLinkSlotMask;
            }
        }
        __syncthreads();
    };
    narrow_gradient_rows<T, kStreaming, false>(x, grads, m, b, lat, lse, logp, runs ? log_domains : 0, Tt, B, A, blank, t0 + wave, 4,
                                        min(t0 + rows_per_group, Tt), s_slot, s_start, s_count, g_slot, stage);
}

template <typename F>
int checked_launch(F&& f)
{
    f();
    return static_cast<int>(hipGetLastError());
}

}  // namespace

namespace {
constexpr int kRowsMaxA = 2048;        // alphabets up to this size use the multi-row kernels

// Rows start on 16-byte boundaries and hold a whole number of 16-byte vectors.
bool vector_ok(const Launch& p)
{
    const int n = (p.dtype == CTC_DTYPE_F32) ? 4 : 8;
    return p.A % n == 0 && reinterpret_cast<uintptr_t>(p.x) % 16 == 0 &&
           reinterpret_cast<uintptr_t>(p.grads) % 16 == 0;
}
}

// Values in the first half of a direction's region, exponents in the second.
static LatticeOut lattice_blocks(const Launch& p)
{
    auto* alpha = reinterpret_cast<uint32_t*>(p.ws + p.lay.alpha);
    auto* beta = reinterpret_cast<uint32_t*>(p.ws + p.lay.beta);
    return {alpha, reinterpret_cast<int*>(alpha + p.lay.ab_doubles), beta, reinterpret_cast<int*>(beta + p.lay.ab_doubles)};
}

int launch_setup(const Launch& p, void* stream)
{
    // (the workers' task list only if the lattice launch has workers; the byte labels after it are read in place)
    const int words = static_cast<int>((p.n_tasks > 0 ? p.lay.labels8 : p.lay.tasks) / 4);
    const unsigned char* labels8 = p.A <= 256 ? static_cast<const unsigned char*>(p.host_image) + p.lay.labels8 : nullptr;
    return checked_launch([&] {
        hipLaunchKernelGGL(ctc_upload_kernel, dim3((words + kRowThreads - 1) / kRowThreads), dim3(kRowThreads),
                           0, static_cast<hipStream_t>(stream), static_cast<const int*>(p.host_image),
                           reinterpret_cast<int*>(p.ws), words, static_cast<int>(p.lay.labels / 4),
                           static_cast<int>(p.lay.tasks / 4), labels8);
    });
}

int launch_plan(const Launch& p, void* stream)
{
    return checked_launch([&] {
        hipLaunchKernelGGL(ctc_plan_kernel, dim3(1), dim3(kPlanThreads), 0, static_cast<hipStream_t>(stream),
                           p.labels, p.dev_label_lengths, p.dev_input_lengths,
                           reinterpret_cast<Utt*>(p.ws + p.lay.meta), reinterpret_cast<int*>(p.ws + p.lay.order),
                           p.dev_status, p.T, p.B, p.A, p.blank, p.max_label, p.poll_budget, p.crowded,
                           p.needs_barrier, p.mode == Mode::kGrad ? 2 : 1);
    });
}

int launch_softmax(const Launch& p, void* stream)
{
    auto* meta = reinterpret_cast<Utt*>(p.ws + p.lay.meta);
    const int* labels = p.labels;
    auto* lse = reinterpret_cast<float*>(p.ws + p.lay.lse);
    auto* emit_blank = reinterpret_cast<float*>(p.ws + p.lay.emit_blank);
    auto* emit_label = reinterpret_cast<float*>(p.ws + p.lay.emit_label);
    const SetupArgs sa{reinterpret_cast<int*>(p.ws + p.lay.links), p.costs,
                       reinterpret_cast<int*>(p.ws + p.lay.chain_err),
                       reinterpret_cast<int*>(p.ws + p.lay.done), reinterpret_cast<int*>(p.ws + p.lay.where),
                       reinterpret_cast<int*>(p.ws + p.lay.leftover), emit_label,
                       reinterpret_cast<double*>(p.ws + p.lay.emit_blank64),
                       p.folded ? nullptr : p.host_flag, p.host_flag_value, p.mode == Mode::kBest,
                       // few utterances: spread each one's grouping over several workgroups (its
                       // latency counts); many: one workgroup each keeps the chip busy already
                       (p.B >= 256 ? 1 : std::max(1, (p.max_label + 63) / 64)) +
                           // (device-resident metadata, narrow alphabets: one more, which builds the utterance's record)
                           (p.folded && p.dev_label_lengths ? 1 : 0)};
    const dim3 block(kRowThreads);
    auto s = static_cast<hipStream_t>(stream);
    const bool f32 = p.dtype == CTC_DTYPE_F32;
    return checked_launch([&] {
        if (p.A <= kDirectMaxA && p.folded) {
            // the smallest alphabets, host metadata: the launch reads the pinned image itself
            const dim3 grid((p.T + kFlagFrames - 1) / kFlagFrames + sa.parts + (p.device_tasks ? 1 : 0), p.B);
            const size_t lds = static_cast<size_t>(kFlagFrames) * p.A * sizeof(float);
            const NarrowImage image{static_cast<const int*>(p.host_image), static_cast<int>(p.lay.labels / 4),
                                    static_cast<int>(p.lay.tasks / 4), static_cast<int>(p.lay.labels8 / 4), p.lay.labels8,
                                    reinterpret_cast<int*>(p.ws + p.lay.labels)};
            auto* row_flags = reinterpret_cast<int*>(p.ws + p.lay.row_flags);
            NarrowArgs args;
            NarrowRows& rows_of = args.rows;
            NarrowDevice dv{};
            if (p.dev_label_lengths) args.plans = plan_table(p.max_label, p.crowded, emission_layout(p.A) == kEmitSymbolMajor);
            if (p.dev_label_lengths)
                dv = NarrowDevice{p.labels, p.dev_label_lengths, p.dev_input_lengths, meta, reinterpret_cast<int*>(p.ws + p.lay.order),
                                  reinterpret_cast<int*>(p.ws + p.lay.status), p.max_label, p.poll_budget,
                                  p.mode == Mode::kGrad ? 2 : 1, p.crowded, p.needs_barrier,
                                  p.device_tasks ? reinterpret_cast<int*>(p.ws + p.lay.tasks) : nullptr, p.share_percent,
                                  p.n_cu % kChainBlock == 0 ? p.n_cu : 0};
            const Utt* records = static_cast<const Utt*>(p.host_image);      // (the host reads its own image)
            for (int b = 0; records && b < p.B; ++b) {
                rows_of.frames[b] = records[b].Tb | ((records[b].flags & kUttRuns) ? kRowsRun : 0) |
                                    ((records[b].flags & kUttGradientLater) ? kRowsGradientLater : 0);
                rows_of.frames_before[b] = records[b].f_off;
                rows_of.label_length[b] = records[b].L;
                rows_of.labels_before[b] = records[b].lab_off;
            }
            if (f32)
                hipLaunchKernelGGL(ctc_softmax_narrow_kernel<float>, grid, block, lds, s, static_cast<const float*>(p.x),
                                   image, reinterpret_cast<int*>(p.ws), lse, emit_blank, emit_label, row_flags, sa,
                                   args, dv, p.T, p.B, p.A, p.blank);
            else
                hipLaunchKernelGGL(ctc_softmax_narrow_kernel<bf16_t>, grid, block, lds, s, static_cast<const bf16_t*>(p.x),
                                   image, reinterpret_cast<int*>(p.ws), lse, emit_blank, emit_label, row_flags, sa,
                                   args, dv, p.T, p.B, p.A, p.blank);
        } else if (p.A <= kDirectMaxA) {
            // the smallest alphabets: 64 frames per workgroup, four lanes per frame, so that a
            // workgroup has several kilobytes under way
            const dim3 grid((p.T + 63) / 64 + sa.parts, p.B);
            const size_t lds = static_cast<size_t>(64) * p.A * sizeof(float);
            if (f32)
                hipLaunchKernelGGL((ctc_softmax_rows_kernel<float, 64>), grid, block, lds, s,
                                   static_cast<const float*>(p.x), meta, labels, lse, emit_blank,
                                   emit_label, sa, p.T, p.B, p.A, p.blank);
            else
                hipLaunchKernelGGL((ctc_softmax_rows_kernel<bf16_t, 64>), grid, block, lds, s,
                                   static_cast<const bf16_t*>(p.x), meta, labels, lse, emit_blank,
                                   emit_label, sa, p.T, p.B, p.A, p.blank);
        } else if (p.A <= 512) {
            const dim3 grid((p.T + 15) / 16 + sa.parts, p.B);
            const size_t lds = static_cast<size_t>(16) * p.A * sizeof(float);
            if (f32)
                hipLaunchKernelGGL((ctc_softmax_rows_kernel<float, 16>), grid, block, lds, s,
                                   static_cast<const float*>(p.x), meta, labels, lse, emit_blank,
                                   emit_label, sa, p.T, p.B, p.A, p.blank);
            else
                hipLaunchKernelGGL((ctc_softmax_rows_kernel<bf16_t, 16>), grid, block, lds, s,
                                   static_cast<const bf16_t*>(p.x), meta, labels, lse, emit_blank,
                                   emit_label, sa, p.T, p.B, p.A, p.blank);
        } else if (p.A <= kRowsMaxA) {
            const dim3 grid((p.T + 3) / 4 + sa.parts, p.B);
            const size_t lds = static_cast<size_t>(4) * p.A * sizeof(float);
            if (f32)
                hipLaunchKernelGGL((ctc_softmax_rows_kernel<float, 4>), grid, block, lds, s,
                                   static_cast<const float*>(p.x), meta, labels, lse, emit_blank,
                                   emit_label, sa, p.T, p.B, p.A, p.blank);
            else
                hipLaunchKernelGGL((ctc_softmax_rows_kernel<bf16_t, 4>), grid, block, lds, s,
                                   static_cast<const bf16_t*>(p.x), meta, labels, lse, emit_blank,
                                   emit_label, sa, p.T, p.B, p.A, p.blank);
        } else if (vector_ok(p) && p.A <= kWideMaxA && p.T + 1 <= kMaxBatch) {
            // (frames index the second grid dimension here, which ends at 65535; longer tensors take
            // the scalar kernel below, whose second dimension is the utterance)
            const dim3 grid(p.B, p.T + 1);
            if (f32)
                hipLaunchKernelGGL(ctc_softmax_wide_kernel<float>, grid, block, 0, s,
                                   static_cast<const float*>(p.x), static_cast<float*>(p.grads), meta, labels, lse, emit_blank,
                                   emit_label, sa, p.T, p.B, p.A, p.blank);
            else
                hipLaunchKernelGGL(ctc_softmax_wide_kernel<bf16_t>, grid, block, 0, s,
                                   static_cast<const bf16_t*>(p.x), static_cast<bf16_t*>(p.grads), meta, labels, lse, emit_blank,
                                   emit_label, sa, p.T, p.B, p.A, p.blank);
        } else {
            const dim3 grid(p.T + 1, p.B);
            if (f32)
                hipLaunchKernelGGL(ctc_softmax_kernel<float>, grid, block, 0, s,
                                   static_cast<const float*>(p.x), static_cast<float*>(p.grads), meta, labels, lse, emit_blank,
                                   emit_label, sa, p.T, p.B, p.A, p.blank);
            else
                hipLaunchKernelGGL(ctc_softmax_kernel<bf16_t>, grid, block, 0, s,
                                   static_cast<const bf16_t*>(p.x), static_cast<bf16_t*>(p.grads), meta, labels, lse, emit_blank,
                                   emit_label, sa, p.T, p.B, p.A, p.blank);
        }
    });
}

int launch_lattice(const Launch& p, void* stream)
{
    // (a call whose softmax launch read the pinned image itself needs this launch for the release, chains or not)
    if (p.n_run == 0 && !(p.folded && p.host_flag)) return 0;
    auto* meta = reinterpret_cast<const Utt*>(p.ws + p.lay.meta);
    auto* order = reinterpret_cast<const int*>(p.ws + p.lay.order);
    const int* labels = p.labels;
    auto* emit_blank = reinterpret_cast<const float*>(p.ws + p.lay.emit_blank);
    auto* emit_label = reinterpret_cast<const float*>(p.ws + p.lay.emit_label);
    auto* sink = reinterpret_cast<uint32_t*>(p.ws + p.lay.sink);
    const LatticeOut lat = lattice_blocks(p);
    auto* logp = reinterpret_cast<double*>(p.ws + p.lay.logp);
    auto* chain_err = reinterpret_cast<int*>(p.ws + p.lay.chain_err);
    size_t lds_bytes = (p.max_waves > 1 && !p.needs_barrier) ? halo_lds_bytes(p.max_waves) : 0;
    int n_groups = std::max(p.n_chains, 1);
    WorkerArgs wk{};
    wk.row_flags = p.folded ? reinterpret_cast<const int*>(p.ws + p.lay.row_flags) : nullptr;
    wk.flag_blocks = (p.T + kFlagFrames - 1) / kFlagFrames;
    wk.domain = reinterpret_cast<int*>(p.ws + p.lay.domain);
    wk.host_flag = p.folded ? p.host_flag : nullptr;
    wk.host_flag_value = p.host_flag_value;
    if (p.folded && p.dev_status) {
        wk.status_words = reinterpret_cast<const int*>(p.ws + p.lay.status);
        wk.status_out = p.dev_status;
        wk.status_count = p.B;
    }
    // Workers (kTaskRows): as many workgroups per idle compute unit as make kWorkerWavesPerCu
    // wavefronts, in rounds of n_cu workgroups whose first n_chains leave at once; their LDS holds
    // the list's table and a piece per wavefront.
    if (p.n_tasks > 0) {
        const size_t table = kXcds + 1 + 3 * static_cast<size_t>(p.n_task_entries) + 1, piece = 2 * static_cast<size_t>(p.max_label) + 129;
        lds_bytes = std::min<size_t>(std::max(lds_bytes, (table + p.max_waves * piece) * 4), 64 << 10);
        const int waves = static_cast<int>(std::min<size_t>(p.max_waves, (lds_bytes / 4 - table) / piece));
        const int idle = p.n_cu - p.n_chains;
        const int per_cu = std::max(1, kWorkerWavesPerCu / p.max_waves);
        // no more workgroups than give every working wavefront a task
        const int rounds = std::max(1, std::min(per_cu, (p.n_tasks + idle * waves - 1) / (idle * waves)));
        n_groups = p.n_cu * rounds;
        wk.x = p.x;
        wk.grads = p.grads;
        wk.links = reinterpret_cast<const int*>(p.ws + p.lay.links);
        wk.lse = reinterpret_cast<const float*>(p.ws + p.lay.lse);
        wk.tasks = reinterpret_cast<const int*>(p.ws + p.lay.tasks);
        wk.done = reinterpret_cast<int*>(p.ws + p.lay.done);
        wk.where = reinterpret_cast<int*>(p.ws + p.lay.where);
        wk.leftover = reinterpret_cast<int*>(p.ws + p.lay.leftover);
        wk.n_tasks = p.n_tasks;
        wk.n_entries = p.device_tasks ? -1 : p.n_task_entries;      // (-1: the list's first block says how many)
        wk.n_chains = p.n_chains;
        wk.n_cu = p.n_cu;
        wk.rounds = rounds;
        wk.worker_waves = waves;
        wk.T = p.T; wk.B = p.B; wk.A = p.A; wk.blank = p.blank; wk.Lmax = p.max_label;
        wk.dtype = static_cast<int>(p.dtype);
        wk.lds_ints = static_cast<int>(lds_bytes / 4);
    }
    const dim3 grid(n_groups), block(64 * p.max_waves);
    auto s = static_cast<hipStream_t>(stream);
#define CTC_LAUNCH_LATTICE(KERNEL)                                                                 \
    hipLaunchKernelGGL(KERNEL, grid, block, lds_bytes, s, meta, order, labels, emit_blank,                 \
                       reinterpret_cast<const double*>(p.ws + p.lay.emit_blank64), emit_label,            \
                       lat, logp, p.costs, chain_err, sink, wk)
    // The emission layout is the launch's (emission_layout), and a template parameter of the kernels.
    const bool symbol_major = emission_layout(p.A) == kEmitSymbolMajor;
#define CTC_LAUNCH_LATTICE_MODE(KERNEL, MODE)                                                       \
    do {                                                                                           \
        if (symbol_major) CTC_LAUNCH_LATTICE((KERNEL<MODE, true>));                                \
        else CTC_LAUNCH_LATTICE((KERNEL<MODE, false>));                                            \
    } while (0)
#define CTC_LAUNCH_LATTICE_KERNEL(KERNEL)                                                           \
    do {                                                                                           \
        if (p.mode == Mode::kLoss) CTC_LAUNCH_LATTICE_MODE(KERNEL, Mode::kLoss);                   \
        else if (p.mode == Mode::kBest) CTC_LAUNCH_LATTICE_MODE(KERNEL, Mode::kBest);              \
        else CTC_LAUNCH_LATTICE_MODE(KERNEL, Mode::kGrad);                                         \
    } while (0)
    return checked_launch([&] {
        // (measurements: the two recursions one after the other, forward chains first, as two launches)
        for (int pass = 0; pass < (p.sequential_chains ? 2 : 1); ++pass) {
            wk.skip_directions = p.sequential_chains ? (pass == 0 ? 2 : 1) : 0;
            if (p.max_waves == 1) CTC_LAUNCH_LATTICE_KERNEL(ctc_lattice_kernel_w1);
            else if (!p.needs_barrier) CTC_LAUNCH_LATTICE_KERNEL(ctc_lattice_kernel);
            else CTC_LAUNCH_LATTICE_KERNEL(ctc_lattice_kernel_barrier);
        }
    });
#undef CTC_LAUNCH_LATTICE_KERNEL
#undef CTC_LAUNCH_LATTICE_MODE
#undef CTC_LAUNCH_LATTICE
}

int launch_backtrace(const Launch& p, void* stream)
{
    auto* meta = reinterpret_cast<const Utt*>(p.ws + p.lay.meta);
    auto* choices = reinterpret_cast<const unsigned char*>(p.ws + p.lay.alpha);
    auto* end_state = reinterpret_cast<const double*>(p.ws + p.lay.logp);
    auto* chain_err = reinterpret_cast<const int*>(p.ws + p.lay.chain_err);
    return checked_launch([&] {
        hipLaunchKernelGGL(ctc_backtrace_kernel, dim3(p.B), dim3(64), 0, static_cast<hipStream_t>(stream),
                           meta, choices, end_state, chain_err, p.costs, p.alignment, p.T);
    });
}

int launch_gradient(const Launch& p, void* stream)
{
    auto* meta = reinterpret_cast<const Utt*>(p.ws + p.lay.meta);
    const int* labels = p.labels;
    auto* links = reinterpret_cast<const int*>(p.ws + p.lay.links);
    auto* lse = reinterpret_cast<const float*>(p.ws + p.lay.lse);
    const LatticeOut lat = lattice_blocks(p);
    auto* logp = reinterpret_cast<const double*>(p.ws + p.lay.logp);
    auto* chain_err = reinterpret_cast<const int*>(p.ws + p.lay.chain_err);
    const dim3 block(kRowThreads);
    auto s = static_cast<hipStream_t>(stream);
    const bool f32 = p.dtype == CTC_DTYPE_F32;
    const int Lmax = p.max_label;
    const bool sparse = p.A > kRowsMaxA;
    // Dense form: 16 rows per workgroup amortise the label staging best once the grid is large;
    // smaller grids finish sooner with twice as many, shorter workgroups (measured on the
    // 64- and 512-utterance minibatches).
    const int rows = sparse ? 4 : (static_cast<int64_t>(p.T) * p.B <= (1 << 17) ? 8 : 16);
    const dim3 grid((p.T + rows - 1) / rows, p.B);
    const size_t lds = (2 * static_cast<size_t>(Lmax) + 4 * (static_cast<size_t>(Lmax) + 1 + (sparse ? 0 : p.A))) * 4;
    if (p.A <= 64) {
        // Both lattice blocks together against what the caches hold (kStreamingLatticeBytes).
        const bool streaming = 2 * p.lay.ab_doubles * sizeof(uint32_t) > kStreamingLatticeBytes;
        const size_t nlds = (static_cast<size_t>(Lmax) + 128 + 4 * (static_cast<size_t>(Lmax) + 1)) * 4;
#define CTC_LAUNCH_NARROW(TYPE, STREAMING)                                                          \
    hipLaunchKernelGGL((ctc_gradient_narrow_kernel<TYPE, STREAMING>), grid, block, nlds, s,         \
                       static_cast<const TYPE*>(p.x), static_cast<TYPE*>(p.grads), meta, labels,    \
                       links, lse, lat, logp, chain_err, p.costs, p.T, p.B, p.A, p.blank,           \
                       Lmax, rows, p.n_tasks > 0 ? reinterpret_cast<const int*>(p.ws + p.lay.leftover) : nullptr,   \
                       reinterpret_cast<const int*>(p.ws + p.lay.domain))
        return checked_launch([&] {
            if (f32 && streaming) CTC_LAUNCH_NARROW(float, true);
            else if (f32) CTC_LAUNCH_NARROW(float, false);
            else if (streaming) CTC_LAUNCH_NARROW(bf16_t, true);
            else CTC_LAUNCH_NARROW(bf16_t, false);
        });
#undef CTC_LAUNCH_NARROW
    }
#define CTC_LAUNCH_GRADIENT(TYPE, SPARSE)                                                          \
    hipLaunchKernelGGL((ctc_gradient_rows_kernel<TYPE, SPARSE>), grid, block, lds, s,               \
                       static_cast<const TYPE*>(p.x), static_cast<TYPE*>(p.grads), meta, labels,     \
                       links, lse, lat, logp, chain_err, p.costs, p.T, p.B, p.A, p.blank, Lmax, rows,               \
                       reinterpret_cast<const float*>(p.ws + p.lay.emit_blank),                                       \
                       reinterpret_cast<const float*>(p.ws + p.lay.emit_label),                                       \
                       reinterpret_cast<const int*>(p.ws + p.lay.domain))
    return checked_launch([&] {
        if (f32 && sparse) CTC_LAUNCH_GRADIENT(float, true);
        else if (f32) CTC_LAUNCH_GRADIENT(float, false);
        else if (sparse) CTC_LAUNCH_GRADIENT(bf16_t, true);
        else CTC_LAUNCH_GRADIENT(bf16_t, false);
    });
#undef CTC_LAUNCH_GRADIENT
}

}  // namespace ctc
