// Part of nms_kernels.hip (included there, inside its anonymous namespace): the paper's rule with eliminated victims dropped from further tests.
#pragma once

// ----------------------------------------------------------------------------- paper's rule, eliminated victims skipped

// Under the paper's rule a box survives iff NO better-ranked box eliminates it (section
// "Algorithm Correctness": V_i is the AND over all j), so a victim that has met one eliminator
// needs no further test -- it goes on eliminating others -- and most victims meet theirs among
// the best-ranked boxes.  One workgroup (16 wavefronts) handles a frame:
//
//   * all boxes of the frame are staged in LDS once (box and, per box, the value the decision
//     needs: its threshold T, or its area for the literal division);
//   * the victims still undecided are a LIST in LDS, in rank order (an entry is the byte offset
//     of the victim's box in the staged table);
//   * the outranking boxes ("candidates") are taken in stages [0,128), [128,256), [256,512) ...:
//     a stage's work is cut into items of (four candidate tiles, a box in each lane of as many
//     register sets) x (16 consecutive list entries, read from LDS as broadcasts, so a victim is
//     fetched once for 256 pair tests) -- two tiles x 32 entries in the first, narrow stages --, handed out
//     to the wavefronts through a counter, so every wavefront has work in every stage however few
//     victims are left; the compare's lane mask != 0 is "this victim has an eliminator";
//   * after a stage the victims ranked before its end that are still alive are survivors, the
//     other alive ones are packed to the front of the list, and a table start[t] = number of
//     entries ranked before 64 t is rebuilt from the list (it tells each candidate group where
//     its victims begin, and where the victims begin that every lane of the group outranks).
//
// No pair is tested that involves a victim eliminated in an earlier stage; the result does not
// depend on the stage bounds, only the amount of work does.
//
// Victims do not depend on each other, so with fewer frames than compute units a frame's victims
// are shared out among several workgroups, each with a list of its own (ranks part, part + parts,
// ...) and the whole frame staged as candidates.  Three kernels share the stages: the table staged
// from the rank step's output (early_exit_kernel), the rank step inside (early_exit_ranked_kernel),
// and frames beyond NMS_SORT_CHUNK boxes, whose table stays in memory (early_exit_wide_kernel).
constexpr int kEarlyWaves = 16;
constexpr int kEarlyThreads = kEarlyWaves * 64;
constexpr int kEarlyFirstStage = 128;                 // candidates of the first stage; each further stage doubles the bound
constexpr int kEarlyItemVictims = 32;                 // most list entries of a work item
constexpr int kEarlyItemPairs = 2 * kEarlyItemVictims; // a work item is 64 x this many pair tests: K tiles x 128 / K entries
constexpr int kEarlyTiles = NMS_SORT_CHUNK / kTile;   // 64

struct EarlyShared {
    float4 box[NMS_SORT_CHUNK];                    // rank order; y scaled by NMS_YSCALE in the y-scaled form
    float aux[NMS_SORT_CHUNK];                     // T, NMS_YSCALE * T, or the area
    int list[NMS_SORT_CHUNK + kEarlyItemVictims];  // undecided victims: 16 * rank, ascending; zeros behind the end
    uint8_t dead[NMS_SORT_CHUNK];                  // by list position: an eliminator was found in this stage
    uint8_t survives[NMS_SORT_CHUNK];              // by rank; written out through `order` when the frame is done
    uint16_t order[NMS_SORT_CHUNK];                // rank -> index in the input
    int start[NMS_MAX_N / kTile + 1];              // start[t] = list entries ranked before 64 t
    int count[4 * kEarlyWaves];                    // packing: entries that go on, per 64 list positions
    int next_item;                                 // the stage's next work item that no wavefront has taken
    int irregular;                                 // some y coordinate rules out the y-scaled form
};

// Frames beyond NMS_SORT_CHUNK boxes ("wide"): the table does not fit LDS.  A workgroup stages only
// its own victims (rank part + parts * i at position i; a list entry is 16 i) and fetches the
// candidate tiles of an item from the ranked table in memory.
struct EarlyWide {
    const float4 *box4;  // ranked boxes
    const float *area;   // and their areas
    double m;            // rounding boundary below the threshold (fast form)
    int part, parts;
};

template <int PAIR>
__device__ __forceinline__ bool early_hit(const float4 v, const float4 cb, float aux, float theta, float y_one)
{
    if (PAIR == kPairFastYScaled) return nms_eliminates_fast_yscaled(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, aux, y_one);
    if (PAIR == kPairFast) return nms_eliminates_fast(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, aux);
    return nms_eliminates_exact(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, aux, theta);
}

// One work item: the list entries [V jb, V jb + V), V = 128 / K, against the K candidate tiles held in
// cb[], aux[].  DIAG: some of the victims are ranked within or before the group, or some of the
// group's tiles do not exist, so a lane counts only when its candidate outranks the victim: its
// entry value (at0 + 1024 i for tile i) is below the victim's (16 x the victim's rank: the entry
// itself, or worked out from it when the list holds positions of a staged share, WIDE).
template <int PAIR, bool DIAG, int K, bool WIDE>
__device__ __forceinline__ void early_item(EarlyShared &sh, int jb, int m, const float4 (&cb)[K], const float (&aux)[K],
                                           int at0, int part, int parts, float theta, float y_one, int lane)
{
    constexpr int V = kEarlyItemPairs / K;
    const int4 *entries = reinterpret_cast<const int4 *>(sh.list + V * jb);
    constexpr int kReads = V / 4;
    unsigned word = 0;  // wave-uniform: bit k = entry V jb + k has an eliminator
    // Every lane reads the same address: broadcasts.  Entries are read two steps ahead and the
    // four victims of step c+1 are fetched before those of step c are tested (the scheduling
    // barriers keep the compiler from sinking the reads to their first use, where every one of
    // them would be waited for in full).
    int4 e[3];
    e[0] = entries[0];
    e[1] = entries[1];
    float4 v[2][4];
    auto fetch = [&](float4 (&dst)[4], const int4 &ent) __attribute__((always_inline)) {
        const char *base = reinterpret_cast<const char *>(sh.box);
        dst[0] = *reinterpret_cast<const float4 *>(base + ent.x);
        dst[1] = *reinterpret_cast<const float4 *>(base + ent.y);
        dst[2] = *reinterpret_cast<const float4 *>(base + ent.z);
        dst[3] = *reinterpret_cast<const float4 *>(base + ent.w);
    };
    fetch(v[0], e[0]);
#pragma unroll
    for (int c = 0; c < kReads; ++c) {
        if (c + 2 < kReads) e[(c + 2) % 3] = entries[c + 2];
        if (c + 1 < kReads) fetch(v[(c + 1) & 1], e[(c + 1) % 3]);
        __builtin_amdgcn_sched_barrier(0);
        const int off[4] = {e[c % 3].x, e[c % 3].y, e[c % 3].z, e[c % 3].w};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            unsigned long long any = 0ull;
            float4 vu = v[c & 1][u];
            // ties this victim's arithmetic to its place between the scheduling barriers (on its own
            // it has no order with respect to them, and instruction selection emits it far ahead)
            asm volatile("" : "+v"(vu.x), "+v"(vu.y), "+v"(vu.z), "+v"(vu.w));
#pragma unroll
            for (int i = 0; i < K; ++i) {
                unsigned long long h = __ballot(early_hit<PAIR>(vu, cb[i], aux[i], theta, y_one));
                // (a tile of the group that does not exist lies at or beyond the end of the frame:
                // no victim is ranked behind any of its lanes, so this test takes it out as well)
                if (DIAG) h &= __ballot(at0 < (WIDE ? off[u] * parts + 16 * part : off[u]) - 16 * kTile * i);
                any |= h;
            }
            // word |= (any != 0) << (4 c + u), written out so that it too stays here and the lane
            // masks are used up at once (left to itself the compiler keeps all of them for later)
            unsigned bit;
            asm volatile("s_cmp_lg_u64 %[any], 0\n\t"
                         "s_cselect_b32 %[bit], %[k], 0\n\t"
                         "s_or_b32 %[word], %[word], %[bit]"
                         : [word] "+s"(word), [bit] "=&s"(bit)
                         : [any] "s"(any), [k] "n"(1u << (4 * c + u))
                         : "scc");
            __builtin_amdgcn_sched_barrier(0);  // one victim at a time: mixing their chains only costs registers
        }
    }
    const int pos = V * jb + lane;
    if (lane < V && ((word >> lane) & 1u) != 0u && pos < m) sh.dead[pos] = 1;
}

// The work items of one stage (candidates [lo, hi), list of m entries) in groups of K tiles.
template <int PAIR, int K, bool WIDE>
__device__ __forceinline__ void early_stage_items(EarlyShared &sh, const EarlyWide &wide, int lo, int hi, int m, int tiles_all,
                                                  float theta, float y_one, int lane, int wave)
{
    constexpr int V = kEarlyItemPairs / K;
    const int groups = ((hi - lo) / kTile + K - 1) / K;  // <= 64

    // lane = candidate group, the last group in lane 0 (its items, most of which straddle the
    // group and cost more, are handed out first; the stage ends on the cheap ones): where the
    // group's victims begin, where those begin that all its lanes outrank, its items
    int p0 = 0, p1 = 0, items = 0;
    if (lane < groups) {
        const int t0 = lo / kTile + K * (groups - 1 - lane);
        p0 = sh.start[t0];
        p1 = sh.start[t0 + K < tiles_all ? t0 + K : tiles_all];
        items = (m + V - 1) / V - p0 / V;
        items = p0 >= m ? 0 : items;
    }
    const int incl = (int)wave_inclusive_sum((unsigned)items);
    const int total = __builtin_amdgcn_readlane(incl, 63);
    int g_held = -1;
    float4 cb[K];
    float aux[K];
    int at0 = 0;
#pragma unroll
    for (int i = 0; i < K; ++i) {
        cb[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        aux[i] = 0.f;
    }
    // items are handed out through a counter (the first one of each wavefront is its own number):
    // an item that straddles the group costs more than one past it, and counts rarely divide evenly
    for (int it = wave; it < total;) {
        int next = 0;
        if (lane == 0) next = __hip_atomic_fetch_add(&sh.next_item, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        const int at = __builtin_amdgcn_readfirstlane(__builtin_popcountll(__ballot(incl <= it)));  // the group's lane
        const int g = groups - 1 - at;
        const int jb = __builtin_amdgcn_readlane(p0, at) / V + (it - __builtin_amdgcn_readlane(incl - items, at));
        const int p1_g = __builtin_amdgcn_readlane(p1, at);
        const int c_lo = lo + K * kTile * g;
        const int tiles = (hi - c_lo) / kTile < K ? (hi - c_lo) / kTile : K;  // of the group that exist
        if (g != g_held) {
#pragma unroll
            for (int i = 0; i < K; ++i) {
                const int c = i < tiles ? c_lo + kTile * i + lane : lane;
                if (WIDE) {
                    cb[i] = wide.box4[c];
                    const float a = wide.area[c];
                    aux[i] = PAIR == kPairExact ? a : nms_pair_threshold(a, wide.m);
                } else {
                    cb[i] = sh.box[c];
                    aux[i] = sh.aux[c];
                }
            }
            at0 = 16 * (c_lo + lane);
            g_held = g;
        }
        if (V * jb < p1_g || tiles < K)
            early_item<PAIR, true, K, WIDE>(sh, jb, m, cb, aux, at0, wide.part, wide.parts, theta, y_one, lane);
        else
            early_item<PAIR, false, K, WIDE>(sh, jb, m, cb, aux, at0, wide.part, wide.parts, theta, y_one, lane);
        it = __builtin_amdgcn_readfirstlane(next);
    }
}

// The initial list of a workgroup's victims, ranks part + parts * i for i < m0 (entry: 16 x the rank,
// or 16 i when only the share is staged), with its start[] table over the frame's tiles_all tiles.
template <bool WIDE>
__device__ __forceinline__ void early_initial_list(EarlyShared &sh, int m0, int part, int parts, int tiles_all)
{
    const int tid = (int)threadIdx.x;
    for (int i = tid; i < NMS_SORT_CHUNK + kEarlyItemVictims; i += kEarlyThreads)
        sh.list[i] = i < m0 ? 16 * (WIDE ? i : part + parts * i) : 0;
    reinterpret_cast<int *>(sh.dead)[tid] = 0;
    reinterpret_cast<int *>(sh.survives)[tid] = 0;
    for (int t = tid; t <= tiles_all; t += kEarlyThreads) {
        const int before = kTile * t > part ? (kTile * t - part + parts - 1) / parts : 0;  // entries ranked before 64 t
        sh.start[t] = before < m0 ? before : m0;
    }
}

// The stages of one frame for the victims of one workgroup: the ranks part, part + parts,
// part + 2 parts ... (victims do not depend on each other, so a frame can be shared out; every
// workgroup needs all the frame's boxes as candidates).  The table is staged, sh.list / sh.dead /
// sh.start describe the initial list of m0 entries and sh.survives is zero.
// WIDE: see EarlyWide (order_f: rank -> input index, in memory); otherwise `wide` only carries part / parts.
template <int PAIR, bool WIDE>
__device__ __forceinline__ void early_exit_frame(EarlyShared &sh, const EarlyWide &wide, int n_f, int m0, float theta, float y_one,
                                                 const int32_t *__restrict__ order_f, uint8_t *__restrict__ keep_f)
{
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int part = wide.part, parts = wide.parts;
    const int staged = (n_f + kTile - 1) / kTile * kTile;
    const int tiles_all = staged / kTile;
    auto rank_of = [&](int entry) __attribute__((always_inline)) { return WIDE ? part + parts * (entry >> 4) : entry >> 4; };
    int m = m0;  // list length
    int lo = 0;
    // Stages double in width, up to 64 groups of four tiles (a lane per group).  A small share is
    // cheap to test and every stage costs its barriers: its stages grow fourfold.
    const int grow = (WIDE && m0 <= 128) || (!WIDE && m0 <= 256) ? 4 : 2;
    for (int bound = kEarlyFirstStage;; bound = grow * bound < bound + 64 * 4 * kTile ? grow * bound : bound + 64 * 4 * kTile) {
        const int hi = bound < staged ? bound : staged;
        const bool last = hi >= n_f;
        if (hi - lo >= 4 * kTile)
            early_stage_items<PAIR, 4, WIDE>(sh, wide, lo, hi, m, tiles_all, theta, y_one, lane, wave);
        else
            early_stage_items<PAIR, 2, WIDE>(sh, wide, lo, hi, m, tiles_all, theta, y_one, lane, wave);
        lds_barrier();

        // Entries still alive: those ranked before `hi` have met every better-ranked box and
        // survive; the others go on, packed to the front.  64 consecutive list positions report
        // how many go on in count[]; a prefix sum gives each its place.
        int entry[4];
        uint8_t gone[4];
        bool on[4];
        unsigned long long on_mask[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {  // all reads first: they do not wait for each other
            const int i = tid + kEarlyThreads * j;
            entry[j] = sh.list[i < m ? i : 0];
            gone[j] = sh.dead[i < m ? i : 0];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = tid + kEarlyThreads * j;
            const bool alive = i < m && gone[j] == 0;
            if (i < m) sh.dead[i] = 0;
            const int r = rank_of(entry[j]);
            if (alive && r < hi) sh.survives[entry[j] >> 4] = 1;
            on[j] = alive && r >= hi;
            on_mask[j] = __ballot(on[j]);
            if (lane == 0) sh.count[kEarlyWaves * j + wave] = __builtin_popcountll(on_mask[j]);
        }
        if (last) break;
        lds_barrier();
        const int mine = sh.count[lane];
        const int upto = (int)wave_inclusive_sum((unsigned)mine);
        const int m_new = __builtin_amdgcn_readlane(upto, 63);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int base = __builtin_amdgcn_readlane(upto - mine, kEarlyWaves * j + wave);
            if (on[j]) sh.list[base + __builtin_popcountll(on_mask[j] & ((1ull << lane) - 1ull))] = entry[j];
        }
        if (tid < kEarlyItemVictims) sh.list[m_new + tid] = 0;
        if (tid == 0) sh.next_item = kEarlyWaves;
        if (m_new == 0) break;
        lds_barrier();
        // start[t] = entries ranked before 64 t: entry i opens every tile after its predecessor's up to its own
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = tid + kEarlyThreads * j;
            if (i < m_new) {
                const int t_cur = rank_of(sh.list[i]) >> 6;
                const int t_prev = i > 0 ? rank_of(sh.list[i - 1]) >> 6 : -1;
                for (int t = t_prev + 1; t <= t_cur; ++t) sh.start[t] = i;
                if (i == m_new - 1)
                    for (int t = t_cur + 1; t <= tiles_all; ++t) sh.start[t] = m_new;
            }
        }
        lds_barrier();
        m = m_new;
        lo = hi;
    }
    lds_barrier();  // every survivor is marked
    for (int i = tid; i < m0; i += kEarlyThreads) {  // `order` is a permutation: each byte once
        const int r = part + parts * i;
        if (WIDE) keep_f[order_f[r]] = sh.survives[i];
        else keep_f[sh.order[r]] = sh.survives[r];
    }
}

// PAIR: kPairFastYScaled (the division-free form of nms_pair.h; a frame with a y coordinate
// outside the y-scaled form's range is staged again as it is and takes the plain fast form) or
// kPairExact (the literal division, for thresholds outside the fast form's range).
template <int PAIR>
__global__ void __launch_bounds__(kEarlyThreads)
early_exit_kernel(const float *__restrict__ sorted5, const int32_t *__restrict__ order,
                  const int32_t *__restrict__ counts, int n_max, int n_pad, int parts, NmsThetaConst th,
                  uint8_t *__restrict__ keep_out)
{
    __shared__ EarlyShared sh;
    const int f = blockIdx.x / parts;
    const int part = blockIdx.x % parts;  // this workgroup's share of the frame's victims
    const int tid = (int)threadIdx.x;
    const int n_f = frame_count(counts, f, n_max);
    const int m0 = n_f > part ? (n_f - part + parts - 1) / parts : 0;
    const float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    const float4 *box4 = reinterpret_cast<const float4 *>(sorted_f);
    const float *area = sorted_f + 4 * (size_t)n_pad;
    uint8_t *keep_f = keep_out + (size_t)f * n_max;
    const int32_t *order_f = order + (size_t)f * n_max;

    if (tid == 0) {
        sh.irregular = 0;
        sh.next_item = kEarlyWaves;
    }
    lds_barrier();
    const int staged = (n_f + kTile - 1) / kTile * kTile;  // padding rows of the table included
    bool odd = false;
    for (int r = tid; r < staged; r += kEarlyThreads) {
        float4 b = box4[r];
        float a = PAIR == kPairExact ? area[r] : nms_pair_threshold(area[r], th.m);
        if (PAIR == kPairFastYScaled) {
            odd |= !(nms_y_regular(b.y) && nms_y_regular(b.w));
            b.y *= NMS_YSCALE;
            b.w *= NMS_YSCALE;
            a *= NMS_YSCALE;
        }
        sh.box[r] = b;
        sh.aux[r] = a;
        sh.order[r] = (uint16_t)(r < n_f ? order_f[r] : 0);
    }
    if (odd) sh.irregular = 1;
    early_initial_list<false>(sh, m0, part, parts, staged / kTile);
    lds_barrier();
    float y_one;  // NMS_YSCALE in a vector register (opaque to the compiler so it stays there)
    asm volatile("v_mov_b32 %0, 0x38800000" : "=v"(y_one));
    const EarlyWide share = {nullptr, nullptr, 0.0, part, parts};
    if (part == 0)
        for (int i = n_f + tid; i < n_max; i += kEarlyThreads) keep_f[i] = 0;
    if (PAIR == kPairFastYScaled && sh.irregular != 0) {
        // some y coordinate is outside the scaled form's range: the table again, as it is, and the plain form
        for (int r = tid; r < staged; r += kEarlyThreads) {  // the rows this thread staged itself
            sh.box[r] = box4[r];
            sh.aux[r] = nms_pair_threshold(area[r], th.m);
        }
        lds_barrier();
        early_exit_frame<kPairFast, false>(sh, share, n_f, m0, th.theta, y_one, nullptr, keep_f);
        return;
    }
    early_exit_frame<PAIR, false>(sh, share, n_f, m0, th.theta, y_one, nullptr, keep_f);
}

// Frames beyond NMS_SORT_CHUNK boxes (see EarlyWide): parts >= n_max / NMS_SORT_CHUNK workgroups
// per frame, each with the victims of ranks part, part + parts, ...; PAIR: kPairFast or kPairExact.
template <int PAIR>
__global__ void __launch_bounds__(kEarlyThreads)
early_exit_wide_kernel(const float *__restrict__ sorted5, const int32_t *__restrict__ order,
                       const int32_t *__restrict__ counts, int n_max, int n_pad, int parts, NmsThetaConst th,
                       uint8_t *__restrict__ keep_out)
{
    __shared__ EarlyShared sh;
    const int f = blockIdx.x / parts;
    const int part = blockIdx.x % parts;
    const int tid = (int)threadIdx.x;
    const int n_f = frame_count(counts, f, n_max);
    const int m0 = n_f > part ? (n_f - part + parts - 1) / parts : 0;  // <= NMS_SORT_CHUNK
    const float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    const EarlyWide wide = {reinterpret_cast<const float4 *>(sorted_f), sorted_f + 4 * (size_t)n_pad, th.m, part, parts};
    uint8_t *keep_f = keep_out + (size_t)f * n_max;

    if (tid == 0) sh.next_item = kEarlyWaves;
    for (int i = tid; i < m0; i += kEarlyThreads) sh.box[i] = wide.box4[part + parts * i];
    early_initial_list<true>(sh, m0, part, parts, (n_f + kTile - 1) / kTile);
    if (part == 0)
        for (int i = n_f + tid; i < n_max; i += kEarlyThreads) keep_f[i] = 0;
    lds_barrier();
    early_exit_frame<PAIR, true>(sh, wide, n_f, m0, th.theta, 0.f, order + (size_t)f * n_max, keep_f);
}

// The same with the rank step inside (frames of more than 2048 boxes, where the rank kernel
// would run with this kernel's 1024 threads anyway): scores and boxes are fetched in input
// order, sorted in LDS (radix_rank_large of rank.h), and go from the registers straight into the
// staged table -- no order / box table in memory, no second launch.  The LDS of the rank step is
// the LDS of the list afterwards.
struct EarlyRankShared {
    unsigned long long keys[NMS_SORT_CHUNK];
    unsigned hist[NMS_SORT_CHUNK];   // one row of 256 digit counts per wavefront
    unsigned wbase[NMS_SORT_CHUNK];  // one row of 256 start offsets per wavefront
    unsigned tot[256];
    float4 stage[NMS_SORT_CHUNK];    // during the sort: the wavefronts' lane-mask tables
};

template <int PAIR>
__global__ void __launch_bounds__(kEarlyThreads)
early_exit_ranked_kernel(const float *__restrict__ boxes, const float *__restrict__ scores,
                         const int32_t *__restrict__ counts, int n_max, NmsThetaConst th, uint8_t *__restrict__ keep_out)
{
    constexpr size_t kBytes = sizeof(EarlyShared) > sizeof(EarlyRankShared) ? sizeof(EarlyShared) : sizeof(EarlyRankShared);
    __shared__ __align__(16) unsigned char raw[kBytes];
    EarlyShared &sh = *reinterpret_cast<EarlyShared *>(raw);
    EarlyRankShared &rk = *reinterpret_cast<EarlyRankShared *>(raw);
    const int f = blockIdx.x;
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63;
    const int n_f = frame_count(counts, f, n_max);
    const float *scores_f = scores + (size_t)f * n_max;
    const float4 *boxes_f = reinterpret_cast<const float4 *>(boxes + (size_t)f * n_max * 4);
    uint8_t *keep_f = keep_out + (size_t)f * n_max;

    int e[4];
    unsigned key32[4], index[4];
    float4 mine[4];  // box e[q] of the input
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        e[q] = (tid >> 6) * 256 + q * 64 + lane;
        const unsigned long long key = e[q] < n_f ? nms_rank_key(scores_f[e[q]], (unsigned)e[q]) : kSentinel;
        key32[q] = (unsigned)(key >> 32);
        index[q] = (unsigned)key;
        mine[q] = e[q] < n_f ? boxes_f[e[q]] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    radix_rank_large<kEarlyWaves>(key32, index, e, rk.keys, rk.hist, rk.tot, rk.wbase, reinterpret_cast<unsigned long long *>(rk.stage));  // ends with a barrier
#pragma unroll
    for (int q = 0; q < 4; ++q) rk.stage[e[q]] = mine[q];
    __syncthreads();
    float4 b[4];  // the box of rank tid + 1024 q, or the padding row (0,0,0,0) of area 1, which eliminates nothing
    int idx[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int r = tid + kEarlyThreads * q;
        idx[q] = r < n_f ? (int)(unsigned)rk.keys[r] : 0;
        b[q] = r < n_f ? rk.stage[idx[q]] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    bool odd = false;
#pragma unroll
    for (int q = 0; q < 4; ++q) odd |= !(nms_y_regular(b[q].y) && nms_y_regular(b[q].w));
    // (a barrier: everything of the rank step is in registers from here on, its LDS is free)
    const bool scaled = PAIR == kPairFastYScaled && __syncthreads_or(odd ? 1 : 0) == 0;
    if (PAIR != kPairFastYScaled) __syncthreads();

    const int staged = (n_f + kTile - 1) / kTile * kTile;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int r = tid + kEarlyThreads * q;
        if (r < staged) {
            const float area = nms_box_area(b[q].x, b[q].y, b[q].z, b[q].w);
            float a = PAIR == kPairExact ? area : nms_pair_threshold(area, th.m);
            float4 bs = b[q];
            if (scaled) {
                bs.y *= NMS_YSCALE;
                bs.w *= NMS_YSCALE;
                a *= NMS_YSCALE;
            }
            sh.box[r] = bs;
            sh.aux[r] = a;
            sh.order[r] = (uint16_t)idx[q];
        }
    }
    if (tid == 0) sh.next_item = kEarlyWaves;
    early_initial_list<false>(sh, n_f, 0, 1, staged / kTile);
    for (int i = n_f + tid; i < n_max; i += kEarlyThreads) keep_f[i] = 0;
    lds_barrier();
    float y_one;  // NMS_YSCALE in a vector register (opaque to the compiler so it stays there)
    asm volatile("v_mov_b32 %0, 0x38800000" : "=v"(y_one));
    const EarlyWide whole = {nullptr, nullptr, 0.0, 0, 1};
    if (PAIR == kPairFastYScaled && !scaled)
        early_exit_frame<kPairFast, false>(sh, whole, n_f, n_f, th.theta, y_one, nullptr, keep_f);
    else
        early_exit_frame<PAIR, false>(sh, whole, n_f, n_f, th.theta, y_one, nullptr, keep_f);
}
