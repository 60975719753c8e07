// rest_retrieve for gfx950: Algorithm 1 (longest matching suffix via the suffix array), continuation
// gather, Algorithm 2 (Trie weights and top-c nodes) and the breadth-first layout with its tree mask
// ("Draft verification") of REST, arXiv 2311.08252 -- one kernel launch, one 1024-thread workgroup per context.
//
// Phase A, search.  Wavefront w looks for the suffix of length n = n_max - w; the fifteen lengths are
// independent searches (a shorter suffix of s is not a prefix of a longer one, so their suffix-array ranges
// do not nest) and run concurrently.  A search is 65-ary: the 64 lanes probe 64 pivots of the current
// rank interval at once and a ballot picks the sub-interval, so 10^8 ranks take 2 LDS levels plus 3 rounds of
// dependent global reads instead of 27.  The two top levels come from a table of 1023 sampled suffix keys
// (first 16 tokens each) that sits in LDS.  Lower and upper bound advance in the same rounds, and a wavefront
// stops as soon as a longer suffix is known to match.
//
// Every probe touches its own cache line, and a compute unit resolves such fully divergent reads at about one
// lane per clock, so the number of load instructions -- not memory latency -- sets the time of a search.  Tokens
// are therefore read four at a time (one 16-byte read at token alignment) and a probe reads on only while it
// still ties with the query.
//
// Phase B, Trie without a Trie.  The kept occurrences are consecutive suffix-array ranks, hence already in
// lexicographic order, so the Trie is implicit in the longest-common-prefix array of adjacent candidates:
// a node at depth d starts at row r iff lcp[r] < d <= len[r], and its weight is the distance to the next row
// with lcp < d.  Per-depth segment-start bitmaps are built with wavefront ballots; everything after that works on
// the bitmaps 64 rows at a time with plain 64-bit logic (eight threads per word): nodes of weight 1 -- nearly all of
// them deep in the Trie -- are counted with a popcount, only heavier nodes are visited one by one.
// Top-c is a three-level counting select on the order (weight desc, depth asc, row asc): weight histogram,
// depth histogram inside the boundary weight, row rank inside the boundary depth.
#include <mutex>

#include "common.h"

namespace {

constexpr int kThreads = 1024;
constexpr int kWavesPerWG = 16;
constexpr int kTopMax = 1023;        // sampled suffix keys cached in LDS
constexpr int kKeyLen = REST_MAX_SUFFIX_LEN;
// Sampled-key table, as int32 words (the same layout in global memory and in LDS):
//   [0, kCoarse)           coarse pivots, token-major: word j * 64 + l = token j of key 16 l + 15
//   [kCoarse, kTabKeys)    suffix-array rank of key k
//   [kTabKeys, ...)        keys in groups of 16, token-major inside a group: word g * 256 + j * 16 + l = token j of
//                          key 16 g + l
// Both levels are read by consecutive lanes at consecutive words, i.e. without LDS bank conflicts.
constexpr int kCoarse = 64 * kKeyLen;
constexpr int kTabKeys = kCoarse + 1024;
__host__ __device__ constexpr int table_words(int top_count) { return kTabKeys + ((top_count + 15) / 16) * 16 * kKeyLen; }

struct RetrieveParams {
    const void* corpus;
    const void* sa;
    const int32_t* top_keys;
    uint64_t n_tokens;
    int32_t top_count;
    const int32_t* contexts;
    const int32_t* ctx_len;
    int32_t ctx_stride;
    int32_t n_max, n_min, K, m, c, mask_words;
    int32_t random_seqs;  // 0, or the number of randomly drawn candidates that replace the kept ones
    uint64_t seed;
    int32_t strided;      // more occurrences than K: keep an evenly spaced sample of the range instead of its head
    rest_tree out;
    // LDS layout of phase B (byte offsets into dynamic LDS)
    int32_t words;        // bitmap words per depth = K/64 + 1
    int32_t off_seg, off_lcp, off_len, off_hist, off_part, off_sel, off_pos, off_after, off_short, off_misc;
};

template <typename TokT>
__device__ inline int32_t load_tok(const void* corpus, uint64_t n, uint64_t pos) {
    return pos < n ? (int32_t)((const TokT*)corpus)[pos] : -1;
}

// entry `rank` of the suffix array of n entries; the entry itself is a position in the stream, i.e. below n
template <typename SaT>
__device__ inline uint32_t load_sa(const void* sa, uint64_t n, uint32_t rank) {
    return (uint32_t)REST_IDX(((const SaT*)sa)[REST_IDX(rank, n, 0)], n, 1);
}

// tokens pos .. pos+3 of the stream with one read (element-wise, -1 past the end, for the last three positions)
template <typename TokT>
__device__ inline void load_tok4(const void* corpus, uint64_t n, uint64_t pos, int32_t (&out)[4]) {
    if (pos + 4 <= n) {
        TokT v[4];
        __builtin_memcpy(v, (const TokT*)corpus + pos, sizeof(v));
#pragma unroll
        for (int j = 0; j < 4; j++) out[j] = (int32_t)v[j];
    } else {
#pragma unroll
        for (int j = 0; j < 4; j++) out[j] = load_tok<TokT>(corpus, n, pos + j);
    }
}

// tokens pos .. pos+N-1 with one read of N tokens (N a power of two), element-wise near the end of the stream
template <typename TokT, int N>
__device__ inline void load_tok_group(const void* corpus, uint64_t n, uint64_t pos, int32_t (&out)[N]) {
    if (pos + N <= n) {
        TokT v[N];
        __builtin_memcpy(v, (const TokT*)corpus + pos, sizeof(v));
#pragma unroll
        for (int j = 0; j < N; j++) out[j] = (int32_t)v[j];
    } else {
#pragma unroll
        for (int j = 0; j < N; j++) out[j] = load_tok<TokT>(corpus, n, pos + j);
    }
}
// tokens of a 16-byte read
template <typename TokT>
constexpr int kWide = 16 / (int)sizeof(TokT);

// Three-way comparison of the first n tokens of two suffixes (at pos1 for lanes with on1, at pos2 for lanes with
// on2) with q; end of stream = -1 < every token.  Tokens are read four at a time and both suffixes' reads are issued
// together.  Most probes differ from q within the first four tokens; the few that tie there read all their remaining
// tokens at once, so that a round costs two dependent reads, not one per group of four.
template <typename TokT>
__device__ inline void cmp_suffix2(const void* corpus, uint64_t ntok, uint32_t pos1, bool on1, uint32_t pos2, bool on2,
                                   const int32_t (&q)[kKeyLen], int n, int& c1, int& c2) {
    c1 = 0;
    c2 = 0;
    auto settle = [&](int g, bool t, const int32_t (&a)[4], int& c) {
#pragma unroll
        for (int j = 3; j >= 0; j--)
            if (t && 4 * g + j < n && a[j] != q[4 * g + j]) c = a[j] < q[4 * g + j] ? -1 : 1;
    };
    {
        int32_t a1[4] = {0, 0, 0, 0}, a2[4] = {0, 0, 0, 0};
        if (on1) load_tok4<TokT>(corpus, ntok, (uint64_t)pos1, a1);
        if (on2) load_tok4<TokT>(corpus, ntok, (uint64_t)pos2, a2);
        settle(0, on1, a1, c1);
        settle(0, on2, a2, c2);
    }
    if (n > 4) {
        const bool t1 = on1 && c1 == 0, t2 = on2 && c2 == 0;
        int32_t a1[kKeyLen / 4][4], a2[kKeyLen / 4][4];
#pragma unroll
        for (int g = 1; g < kKeyLen / 4; g++) {
#pragma unroll
            for (int j = 0; j < 4; j++) a1[g][j] = a2[g][j] = 0;
            if (4 * g < n) {
                if (t1) load_tok4<TokT>(corpus, ntok, (uint64_t)pos1 + 4 * g, a1[g]);
                if (t2) load_tok4<TokT>(corpus, ntok, (uint64_t)pos2 + 4 * g, a2[g]);
            }
        }
        // the first group that differs decides: later groups only speak while the earlier ones tie
#pragma unroll
        for (int g = 1; g < kKeyLen / 4; g++) {
            if (4 * g < n) {
                settle(g, t1 && c1 == 0, a1[g], c1);
                settle(g, t2 && c2 == 0, a2[g], c2);
            }
        }
    }
}

__device__ inline int popc64(uint64_t x) { return __popcll(x); }

// Bracket of one bound: ranks below `a` lie under the bound, ranks from `b` on do not; closed when a == b.
struct Bracket {
    uint32_t a, b;
    __device__ bool open() const { return a < b; }
    // 64 probes of an open bracket, increasing in the lane index: every rank if it holds at most 64, else pivots
    __device__ uint32_t probe(int lane, bool& real) const {
        const uint32_t len = b - a;
        const bool fine = len <= 64;
        real = !fine || (uint32_t)lane < len;
        return fine ? a + lane : a + (uint32_t)(((uint64_t)len * (lane + 1)) / 65);
    }
    // k of the n_real probes (ranks r, increasing over the first n_real lanes) lie under the bound
    __device__ void tighten(uint32_t r, int k, int n_real) {
        const uint32_t below = __shfl(r, k > 0 ? k - 1 : 0, 64), at = __shfl(r, k < n_real ? k : 0, 64);
        if (k > 0 && below + 1 > a) a = below + 1;
        if (k < n_real && at < b) b = at;
    }
};

// One wavefront: [lo, hi) = ranks of the suffixes whose first n tokens equal q.  `best` (LDS) is the smallest
// wavefront index known to have a match: a wavefront with a larger index (a shorter suffix) stops as soon as it
// sees a smaller one there and reports an empty range, which the caller never selects.
template <typename TokT, typename SaT>
__device__ __forceinline__ void wave_search(const RetrieveParams& p, const int32_t* lds_tab, const int32_t (&q)[kKeyLen], int n,
                            int wave, int32_t* best, uint32_t& out_lo, uint32_t& out_hi) {
    const int lane = threadIdx.x & 63;
    const uint32_t N = (uint32_t)p.n_tokens;
    const int tc = p.top_count;
    // ---- two levels in LDS: 64 coarse pivots (every 16th sampled key), then the 15 keys of one group
    const int32_t* coarse = lds_tab;
    const uint32_t* rank = (const uint32_t*)(lds_tab + kCoarse);
    const int32_t* keys = lds_tab + kTabKeys;
    // token j of the key at col[j * stride]; front to back, and only while some lane's key still ties with q: keys
    // spread over a rank interval mostly differ from q within a few tokens
    auto cmp_word = [&](const int32_t* col, int stride) {
        int c = 0;
#pragma unroll
        for (int j = 0; j < kKeyLen; j++) {
            if (j >= n || __ballot(c == 0) == 0) break;
            const int32_t x = col[j * stride];
            if (c == 0 && x != q[j]) c = x < q[j] ? -1 : 1;
        }
        return c;
    };
    int cnt_lt = 0, cnt_le = 0;
    if (tc > 0) {
        const int c = 16 * lane + 15 < tc ? cmp_word(coarse + lane, 64) : 1;
        const int g_lt = popc64(__ballot(c < 0)), g_le = popc64(__ballot(c <= 0));
        const int c1 = (lane < 15 && 16 * g_lt + lane < tc) ? cmp_word(keys + g_lt * 256 + lane, 16) : 1;
        cnt_lt = 16 * g_lt + popc64(__ballot(c1 < 0));
        int c2 = c1;
        if (g_le != g_lt) c2 = (lane < 15 && 16 * g_le + lane < tc) ? cmp_word(keys + g_le * 256 + lane, 16) : 1;
        cnt_le = 16 * g_le + popc64(__ballot(c2 <= 0));
        if (cnt_le > cnt_lt && lane == 0) atomicMin(best, wave);      // a sampled key equals q
    }
    // lower bound: ranks under it compare <; upper bound: ranks under it compare <=
    Bracket lo, hi;
    lo.a = cnt_lt ? rank[cnt_lt - 1] + 1 : 0;
    lo.b = cnt_lt < tc ? rank[cnt_lt] : N;
    hi.a = cnt_le ? rank[cnt_le - 1] + 1 : 0;
    hi.b = cnt_le < tc ? rank[cnt_le] : N;

    // Global rounds.  A round probes the lower bound's bracket and, when it is a different interval, the upper
    // bound's bracket too; the reads of both probe sets are in flight together and every probe tightens both
    // brackets, so the two bounds cost the rounds of the slower one.
    while (lo.open() || hi.open()) {
        if (*(volatile int32_t*)best < wave) {
            out_lo = out_hi = 0;
            return;
        }
        const bool go1 = lo.open();
        const bool go2 = hi.open() && !(go1 && hi.a == lo.a && hi.b == lo.b);
        bool real1 = false, real2 = false;
        uint32_t r1 = 0, r2 = 0;
        if (go1) r1 = lo.probe(lane, real1);
        if (go2) r2 = hi.probe(lane, real2);
        uint32_t pos1 = 0, pos2 = 0;
        if (real1) pos1 = load_sa<SaT>(p.sa, p.n_tokens, r1);
        if (real2) pos2 = load_sa<SaT>(p.sa, p.n_tokens, r2);
        int c1, c2;
        cmp_suffix2<TokT>(p.corpus, p.n_tokens, pos1, real1, pos2, real2, q, n, c1, c2);
        if (__ballot((real1 && c1 == 0) || (real2 && c2 == 0)) && lane == 0) atomicMin(best, wave);
        if (go1) {
            const int n_real = popc64(__ballot(real1));
            const int k_lt = popc64(__ballot(real1 && c1 < 0)), k_le = popc64(__ballot(real1 && c1 <= 0));
            lo.tighten(r1, k_lt, n_real);
            hi.tighten(r1, k_le, n_real);
        }
        if (go2) {
            const int n_real = popc64(__ballot(real2));
            const int k_lt = popc64(__ballot(real2 && c2 < 0)), k_le = popc64(__ballot(real2 && c2 <= 0));
            lo.tighten(r2, k_lt, n_real);
            hi.tighten(r2, k_le, n_real);
        }
    }
    out_lo = lo.a;
    out_hi = hi.a > lo.a ? hi.a : lo.a;
}

// One item = the 64 rows of word wi at depth d, handled by ONE thread with 64-bit bit operations: `node` = rows that
// start a Trie node (a segment start on a row long enough), `ones` = the nodes of weight 1 (the next row starts a
// segment too), `big` = the others.  Deep in the Trie nearly every node has weight 1, so an item is mostly a few
// logic operations and a popcount; only the `big` nodes are visited one by one.
struct Item {
    uint64_t word, node, ones, big;
    int32_t after;      // first segment start in any later word
};
__device__ inline Item classify(const uint64_t* seg, const int32_t* after, const uint64_t* shortbm, const uint8_t* rlen,
                                int words, int row_words, int d, int wi, int R) {
    Item it;
    it.word = seg[(d - 1) * words + wi];
    it.after = after[(d - 1) * words + wi];
    const int left = R - wi * 64;                                   // valid rows in this word
    const uint64_t vmask = left >= 64 ? ~0ull : (left > 0 ? (1ull << left) - 1ull : 0ull);
    it.node = it.word & vmask;
    uint64_t cut = shortbm[wi] & it.node;                           // rows cut short by the end of the stream: rare
    while (cut) {
        const int b = __builtin_ctzll(cut);
        cut &= cut - 1;
        if (rlen[wi * 64 + b] < d) it.node &= ~(1ull << b);
    }
    // a valid row is never the last bit that matters: the terminator rows follow it, in this word or the next
    const uint64_t next0 = wi + 1 < row_words ? seg[(d - 1) * words + wi + 1] & 1ull : 0ull;
    const uint64_t follows = (it.word >> 1) | (next0 << 63);
    it.ones = it.node & follows;
    it.big = it.node & ~follows;
    return it;
}
// weight of the node at bit b of an item: distance to the next segment start
__device__ inline int bit_weight(const Item& it, int wi, int b) {
    const uint64_t later = b < 63 ? it.word & (~0ull << (b + 1)) : 0ull;
    return later ? __builtin_ctzll(later) - b : it.after - (wi * 64 + b);
}

// Entry of the suffix array that holds kept candidate i of the range [lo, lo + S): the first K entries, or, sampling
// S > K occurrences evenly, entry lo + floor(i*S/K) = lo + i*(S/K) + floor(i*(S%K)/K); i and S%K are below K <= 8192,
// so 32 bits hold the product.
__device__ inline uint32_t kept_rank(uint32_t lo, uint32_t S, uint32_t K, bool strided, uint32_t i) {
    if (strided && S > K) return lo + i * (S / K) + (i * (S % K)) / K;
    return lo + i;
}

// One candidate row: the up to m tokens that follow the n_star matched ones at suffix-array entry `entry` (-1 beyond
// the row's end), and how many there are.
template <int kM, typename TokT>
__device__ __forceinline__ void load_row_at(const RetrieveParams& p, const uint32_t start, const bool on, const int n_star,
                                            int32_t (&tok)[kM], int& len) {
    len = 0;
#pragma unroll
    for (int j = 0; j < kM; j++) tok[j] = -1;
    if (on) {
        const uint64_t pos = (uint64_t)start + n_star;
        const uint64_t left = p.n_tokens > pos ? p.n_tokens - pos : 0;
        len = left < (uint64_t)p.m ? (int)left : p.m;
        constexpr int G = kWide<TokT>;                 // 16 bytes a read
#pragma unroll
        for (int g = 0; g < kM / G; g++) {
            int32_t a[G];
#pragma unroll
            for (int j = 0; j < G; j++) a[j] = -1;
            if (G * g < p.m) load_tok_group<TokT, G>(p.corpus, p.n_tokens, pos + G * g, a);
#pragma unroll
            for (int j = 0; j < G; j++) tok[G * g + j] = a[j];
        }
    }
}
template <int kM, typename TokT, typename SaT>
__device__ __forceinline__ void load_row(const RetrieveParams& p, const uint32_t entry, const bool on, const int n_star,
                                         int32_t (&tok)[kM], int& len) {
    const uint32_t start = on ? load_sa<SaT>(p.sa, p.n_tokens, entry) : 0u;
    load_row_at<kM, TokT>(p, start, on, n_star, tok, len);
}

// LDS of the phase B for few rows (byte offsets; the key table is dead by then)
constexpr int kFewTokStride = REST_MAX_CONT_LEN + 1;                 // words per row: odd, so that rows fall on different banks
constexpr int kFewTok = 0;                                           // int32 [64][kFewTokStride]
constexpr int kFewLcp = kFewTok + 64 * kFewTokStride * 4;            // uint8 [64]
constexpr int kFewLen = kFewLcp + 64;                                // uint8 [64]
constexpr int kFewHist = kFewLen + 64;                               // uint32 [65], bin w = nodes of weight w
constexpr int kFewDepth = kFewHist + 65 * 4 + 4;                     // uint32 [64]: per depth, nodes of the boundary weight
constexpr int kFewKept = kFewDepth + 64 * 4;                         // uint32 [64]: per depth, kept nodes
constexpr int kFewTotal = kFewKept + 64 * 4;                         // uint32 [2]
constexpr int kFewSeg = kFewTotal + 8;                               // uint64 [REST_MAX_CONT_LEN] segment starts per depth
constexpr int kFewKeep = kFewSeg + REST_MAX_CONT_LEN * 8;            // uint64 [REST_MAX_CONT_LEN] kept rows per depth
constexpr int kFewNode = kFewKeep + REST_MAX_CONT_LEN * 8;           // uint32 [REST_MAX_NODES]: depth | row << 8 | weight << 16
constexpr int kFewBytes = kFewNode + REST_MAX_NODES * 4;
static_assert(kFewSeg % 8 == 0, "64-bit words are aligned");

// Phase B for at most 64 kept rows -- most contexts: a long suffix matches in a handful of places.  Rows sit in
// lanes, depths in wavefronts (wavefront w takes depths w + 1 and w + 17), so every step is a few instructions per
// wavefront between two barriers and nothing loops over rows or depths:
//   B_d, the segment starts of depth d (rows >= R count as starts), is a ballot; the weight of node (d, r) is the
//   distance to the next set bit of B_d; the boundary weight comes from a 64-bin histogram, the boundary depth from
//   per-depth counts, the row rank inside it from a ballot; the breadth-first slot of a kept node is the number of
//   kept nodes of smaller depth plus those of its own depth in lower rows, so nothing is sorted; the parent of
//   (d, r) is the last set bit of B_{d-1} at or below r; and node a is on the root path of node x iff
//   depth(a) <= depth(x) and row(a) <= row(x) < row(a) + weight(a), which makes a mask word a ballot over 64 slots.
// The rows come from the wavefront `owner` (registers tok / len, lane = row).  Same order and output as the general path.
template <int kM>
__device__ __forceinline__ void few_rows_tree(const RetrieveParams& p, unsigned char* lds, const int b, const int R, const int n_star,
                                              const uint32_t match_count, const int owner, const int32_t (&tok)[kM], const int len) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane;
    const int m = p.m, c = p.c;
    int32_t* o_tok = p.out.draft_tokens + (int64_t)b * c;
    int32_t* o_par = p.out.parent_idx + (int64_t)b * c;
    int32_t* o_pos = p.out.pos_ids + (int64_t)b * c;
    int32_t* o_wgt = p.out.node_weight + (int64_t)b * c;
    uint64_t* o_mask = p.out.tree_mask + (int64_t)b * c * p.mask_words;
    int32_t* l_tok = (int32_t*)(lds + kFewTok);
    uint8_t* l_lcp = lds + kFewLcp;
    uint8_t* l_len = lds + kFewLen;
    uint32_t* l_hist = (uint32_t*)(lds + kFewHist);
    uint32_t* l_depth = (uint32_t*)(lds + kFewDepth);
    uint32_t* l_kept = (uint32_t*)(lds + kFewKept);
    uint32_t* l_total = (uint32_t*)(lds + kFewTotal);
    uint64_t* l_seg = (uint64_t*)(lds + kFewSeg);
    uint64_t* l_keep = (uint64_t*)(lds + kFewKeep);
    uint32_t* l_node = (uint32_t*)(lds + kFewNode);

    // ---- the owner parks its rows and their common prefixes with the previous row; the others clear the counters
    if (wave == owner) {
        int l = 0;
        const int plen = __shfl_up(len, 1, 64);
        bool run = true;
#pragma unroll
        for (int j = 0; j < kM; j++) {
            if (j < m) {
                const int32_t prev = __shfl_up(tok[j], 1, 64);
                run = run && j < len && j < plen && prev == tok[j];
                l += run ? 1 : 0;
                l_tok[r * kFewTokStride + j] = tok[j];
            }
        }
        if (r == 0) l = 0;
        l_lcp[r] = (uint8_t)l;
        l_len[r] = (uint8_t)len;
    } else if (wave == ((owner + 1) & 15)) {
        l_hist[lane] = 0;
        l_depth[lane] = 0;
        l_kept[lane] = 0;
        if (lane < 2) { l_hist[64 + lane] = 0; l_total[lane] = 0; }
    }
    __syncthreads();

    // ---- my depths: segment starts, node weights
    const uint64_t lt = (1ull << r) - 1ull;              // rows below mine
    const uint64_t le = lt | (1ull << r);                // ... and mine
    const int l = l_lcp[r], rl = l_len[r];
    int wgt[2] = {0, 0};
#pragma unroll
    for (int h = 0; h < 2; h++) {
        const int d = wave + 1 + 16 * h;
        if (d <= m) {
            const uint64_t Bd = __ballot(r >= R || l < d);
            const bool node = r < R && l < d && d <= rl;
            const uint64_t later = Bd & ~le;
            const int next = later ? __builtin_ctzll(later) : 64;
            wgt[h] = node ? next - r : 0;
            if (node) atomicAdd(&l_hist[wgt[h]], 1u);
            const uint32_t nodes = (uint32_t)popc64(__ballot(node));
            if (lane == 0) {
                l_seg[d - 1] = Bd;
                atomicAdd(&l_total[0], nodes);
            }
        }
    }
    __syncthreads();

    // ---- boundary of the top c in the order (weight down, depth up, row up)
    const bool take_all = (int)l_total[0] <= c;
    int w_star = 0, d_star = m + 1, need_d = 0;
    uint64_t eq[2] = {0, 0};
    if (!take_all) {                                      // the same for every wavefront
        uint32_t x = l_hist[lane + 1];                    // lane i: weight i + 1 -> after the scan, nodes of weight >= i + 1
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t y = __shfl_down(x, off, 64);
            if (lane + off < 64) x += y;
        }
        const uint64_t enough = __ballot(x >= (uint32_t)c);        // lane 0 holds the total, which is above c
        const int top = 63 - __builtin_clzll(enough);
        w_star = top + 1;
        const int above = top < 63 ? (int)__shfl(x, top + 1, 64) : 0;
        const int need_w = c - above;                     // nodes of the boundary weight to take
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int d = wave + 1 + 16 * h;
            if (d <= m) {
                eq[h] = __ballot(wgt[h] == w_star);
                if (lane == 0) l_depth[d - 1] = (uint32_t)popc64(eq[h]);
            }
        }
        __syncthreads();
        // lane i: nodes of the boundary weight at depth i + 1 -> with the scan, at depths <= i + 1
        const uint32_t v = lane < m ? l_depth[lane] : 0;
        uint32_t y = v;
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t z = __shfl_up(y, off, 64);
            if (lane >= off) y += z;
        }
        const uint64_t reached = __ballot(y >= (uint32_t)need_w);  // not empty: the boundary weight has need_w nodes
        const int at = __builtin_ctzll(reached);
        d_star = at + 1;
        need_d = need_w - (int)(__shfl(y, at, 64) - __shfl(v, at, 64));
    }
    // ---- kept nodes of my depths
    bool keep[2] = {false, false};
    uint64_t Kd[2] = {0, 0};
#pragma unroll
    for (int h = 0; h < 2; h++) {
        const int d = wave + 1 + 16 * h;
        if (d <= m) {
            const int w = wgt[h];
            keep[h] = w > 0 && (take_all || w > w_star ||
                                (w == w_star && (d < d_star || (d == d_star && popc64(eq[h] & lt) < need_d))));
            Kd[h] = __ballot(keep[h]);
            if (lane == 0) {
                l_keep[d - 1] = Kd[h];
                l_kept[d - 1] = (uint32_t)popc64(Kd[h]);
            }
        }
    }
    __syncthreads();

    // ---- slots: lane i first holds the kept nodes of depth i + 1, then those of smaller depths
    int T;
    {
        const uint32_t v = lane < m ? l_kept[lane] : 0;
        uint32_t y = v;
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t z = __shfl_up(y, off, 64);
            if (lane >= off) y += z;
        }
        T = (int)__shfl(y, 63, 64);
        const uint32_t before = y - v;
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int d = wave + 1 + 16 * h;
            if (d <= m) {
                const int first = (int)__shfl(before, d - 1, 64);
                const int first_up = d > 1 ? (int)__shfl(before, d - 2, 64) : 0;
                if (keep[h]) {
                    const int slot = (int)REST_IDX(first + popc64(Kd[h] & lt), c, 5);
                    int par = -1;
                    if (d > 1) {
                        const uint64_t Bu = l_seg[d - 2], Ku = l_keep[d - 2];
                        const int rp = 63 - __builtin_clzll(Bu & le);     // row 0 starts a segment at every depth
                        if ((Ku >> rp) & 1ull) par = first_up + popc64(Ku & ((1ull << rp) - 1ull));
                    }
                    o_tok[slot] = l_tok[r * kFewTokStride + d - 1];
                    o_par[slot] = par;
                    o_pos[slot] = d;
                    o_wgt[slot] = wgt[h];
                    l_node[slot] = (uint32_t)d | ((uint32_t)r << 8) | ((uint32_t)wgt[h] << 16);
                }
            }
        }
    }
    for (int i = T + tid; i < c; i += kThreads) {
        o_tok[i] = -1; o_par[i] = -1; o_pos[i] = 0; o_wgt[i] = 0;
        for (int k = 0; k < p.mask_words; k++) o_mask[(int64_t)i * p.mask_words + k] = 0;
    }
    if (tid == 0) {
        p.out.n_nodes[b] = T;
        p.out.matched_len[b] = n_star;
        p.out.match_count[b] = (int64_t)match_count;
    }
    __syncthreads();

    // ---- mask rows: lanes = the 64 slots of a word
    for (int x = wave; x < T; x += kWavesPerWG) {
        const uint32_t nx = l_node[x];
        const int dx = (int)(nx & 0xffu), rx = (int)((nx >> 8) & 0xffu);
        for (int k = 0; k < p.mask_words; k++) {
            const int a = 64 * k + lane;
            bool on_path = false;
            if (a < T) {
                const uint32_t na = l_node[a];
                const int da = (int)(na & 0xffu), ra = (int)((na >> 8) & 0xffu), wa = (int)(na >> 16);
                on_path = da <= dx && ra <= rx && rx < ra + wa;
            }
            const uint64_t word = __ballot(on_path);
            if (lane == 0) o_mask[(int64_t)x * p.mask_words + k] = word;
        }
    }
}

template <typename TokT, typename SaT>
__global__ __launch_bounds__(kThreads) void retrieve_kernel(RetrieveParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ uint32_t s_lo[kWavesPerWG], s_hi[kWavesPerWG];
    __shared__ int32_t s_best;       // smallest wave index known to have a match: the suffix length chosen in the end
    __shared__ int32_t s_misc[16];

    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t* s = p.contexts + (int64_t)b * p.ctx_stride;
    int t = p.ctx_len[b];
    t = t < 0 ? 0 : (t > p.ctx_stride ? p.ctx_stride : t);

    // ---------------- phase A: the sampled-key table goes to LDS, then one search per wavefront.
    // The reads are issued in this order: the context length (above), my share of the table (into registers), and --
    // once the length is here -- my query tokens; the table is parked in LDS while the query is still on its way, so
    // that the search does not start with a cold read of its own.
    const int32_t* lds_tab = (const int32_t*)lds;
    const int n = p.n_max - wave;
    int32_t q[kKeyLen];
    bool searching;
    {
        constexpr int kShare = (table_words(kTopMax) / 4 + kThreads - 1) / kThreads;
        const int4* src = (const int4*)p.top_keys;
        int4* dst = (int4*)lds;
        const int nvec = table_words(p.top_count) / 4;
        int4 share[kShare];
#pragma unroll
        for (int i = 0; i < kShare; i++) {
            share[i] = make_int4(0, 0, 0, 0);
            if (tid + i * kThreads < nvec) share[i] = src[tid + i * kThreads];
        }
        searching = n >= p.n_min && n <= t;
#pragma unroll
        for (int j = 0; j < kKeyLen; j++) q[j] = (searching && j < n) ? s[t - n + j] : 0;
#pragma unroll
        for (int i = 0; i < kShare; i++)
            if (tid + i * kThreads < nvec) dst[tid + i * kThreads] = share[i];
        if (tid == 0) s_best = kWavesPerWG;
    }
    __syncthreads();
    // A wavefront whose range is small enough for the few-rows phase B requests its rows right away (lane = row): they
    // are on their way while the other searches finish.
    int32_t row_tok[16];
    int row_len = 0;
    bool have_rows = false;
#pragma unroll
    for (int j = 0; j < 16; j++) row_tok[j] = -1;
    {
        uint32_t lo = 0, hi = 0;
        if (searching) wave_search<TokT, SaT>(p, lds_tab, q, n, wave, &s_best, lo, hi);
        {
            const uint32_t S = hi - lo, Rw = S < (uint32_t)p.K ? S : (uint32_t)p.K;
            if (hi > lo && p.random_seqs == 0 && p.m <= 16 && Rw <= 64) {
                load_row<16, TokT, SaT>(p, kept_rank(lo, S, (uint32_t)p.K, p.strided != 0, (uint32_t)lane), (uint32_t)lane < Rw, n,
                                        row_tok, row_len);
                have_rows = true;
            }
        }
        if (lane == 0) {
            s_lo[wave] = lo;
            s_hi[wave] = hi;
            if (hi > lo) atomicMin(&s_best, wave);         // wave 0 holds the longest suffix
        }
    }
    __syncthreads();

    // ---------------- outputs of this context
    const int c = p.c;
    int32_t* o_tok = p.out.draft_tokens + (int64_t)b * c;
    int32_t* o_par = p.out.parent_idx + (int64_t)b * c;
    int32_t* o_pos = p.out.pos_ids + (int64_t)b * c;
    int32_t* o_wgt = p.out.node_weight + (int64_t)b * c;
    uint64_t* o_mask = p.out.tree_mask + (int64_t)b * c * p.mask_words;

    const int sel = s_best < kWavesPerWG ? s_best : -1;
    if (sel < 0) {
        for (int i = tid; i < c; i += kThreads) { o_tok[i] = -1; o_par[i] = -1; o_pos[i] = 0; o_wgt[i] = 0; }
        for (int i = tid; i < c * p.mask_words; i += kThreads) o_mask[i] = 0;
        if (tid == 0) { p.out.n_nodes[b] = 0; p.out.matched_len[b] = 0; p.out.match_count[b] = 0; }
        return;
    }
    const int n_star = p.n_max - sel;
    const uint32_t lo = s_lo[sel], hi = s_hi[sel];
    int R = (int)((hi - lo) < (uint32_t)p.K ? (hi - lo) : (uint32_t)p.K);

    // Random-selection strategy of the ablation: a few drawn candidates take the place of the R kept ones.  Row r of
    // phase B is then kept candidate s_pick[r]; the drawn candidates are sorted, so rows stay in suffix order.
    __shared__ int32_t s_pick[64];
    __shared__ int32_t s_npick;
    const bool drawn = p.random_seqs > 0;
    if (drawn) {
        if (wave == 0) {
            const uint64_t G = 0x9E3779B97F4A7C15ull;
            auto mix = [](uint64_t z) {
                z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
                z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
                return z ^ (z >> 31);
            };
            const uint64_t h = mix(p.seed + G * (uint64_t)(1 + b));
            const bool active = lane < p.random_seqs;
            const uint32_t r = active ? (uint32_t)__umul64hi(mix(h + G * (uint64_t)(1 + lane)), (uint64_t)R) : 0xffffffffu;
            bool first = active;          // no lower lane drew the same candidate
            for (int k = 0; k < 64; k++) {
                const uint32_t o = __shfl(r, k, 64);
                if (k < lane && o == r) first = false;
            }
            int rank = 0;                 // distinct candidates below mine
            for (int k = 0; k < 64; k++) {
                const uint32_t o = __shfl(r, k, 64);
                const int of = __shfl((int)first, k, 64);
                if (of && o < r) rank++;
            }
            if (first) s_pick[rank] = (int32_t)r;
            const int n_first = __popcll(__ballot(first));
            if (lane == 0) s_npick = n_first;
        }
        __syncthreads();
        R = s_npick;
    }
    const int m = p.m;
    const int words = p.words;
    // Kept candidate i is entry lo + i of the suffix array, or, sampling S > K occurrences evenly, entry
    // lo + floor(i*S/K) = lo + i*(S/K) + floor(i*(S%K)/K); i and S%K are below K <= 8192, so 32 bits hold the product.
    const uint32_t S = hi - lo;
    const bool spaced = p.strided != 0 && S > (uint32_t)p.K;
    const uint32_t step_q = spaced ? S / (uint32_t)p.K : 1u, step_r = spaced ? S % (uint32_t)p.K : 0u;
    auto kept_entry = [&](int r) -> uint32_t {
        const uint32_t i = drawn ? (uint32_t)s_pick[r] : (uint32_t)r;
        return spaced ? lo + i * step_q + (i * step_r) / (uint32_t)p.K : lo + i;
    };

    if (R <= 64) {
        // every wavefront is past the search: the key table in LDS is dead
        if (m <= 16) {
            if (wave == sel && !have_rows) load_row<16, TokT, SaT>(p, kept_entry(lane), lane < R, n_star, row_tok, row_len);
            few_rows_tree<16>(p, lds, b, R, n_star, hi - lo, sel, row_tok, row_len);
        } else {
            int32_t tok[REST_MAX_CONT_LEN];
            int len;
            load_row<REST_MAX_CONT_LEN, TokT, SaT>(p, kept_entry(lane), wave == sel && lane < R, n_star, tok, len);
            few_rows_tree<REST_MAX_CONT_LEN>(p, lds, b, R, n_star, hi - lo, sel, tok, len);
        }
        return;
    }

    // ---------------- phase B LDS (aliases the key table, which is dead now)
    uint64_t* seg = (uint64_t*)(lds + p.off_seg);        // [m][words] segment-start bits per depth
    uint8_t* lcp = (uint8_t*)(lds + p.off_lcp);          // [K]
    uint8_t* rlen = (uint8_t*)(lds + p.off_len);         // [K]
    uint32_t* hist = (uint32_t*)(lds + p.off_hist);      // [K + 1] nodes per weight
    uint32_t* part = (uint32_t*)(lds + p.off_part);      // [1024] scan scratch
    uint32_t* sel_key = (uint32_t*)(lds + p.off_sel);    // [c] (depth << 16 | row), then sorted
    uint32_t* sel_wgt = sel_key + REST_MAX_NODES;        // [c]
    uint32_t* srt_key = sel_wgt + REST_MAX_NODES;        // [c]
    uint32_t* srt_wgt = srt_key + REST_MAX_NODES;        // [c]
    uint32_t* rowpos = (uint32_t*)(lds + p.off_pos);     // [K] suffix-array entry of each kept row
    int32_t* after = (int32_t*)(lds + p.off_after);      // [m][words] first set bit of seg[d] in any word after this one
    uint64_t* shortbm = (uint64_t*)(lds + p.off_short);  // [words] rows cut short by the end of the stream

    for (int i = tid; i <= p.K; i += kThreads) hist[i] = 0;
    if (tid < 16) s_misc[tid] = 0;

    // ---- B1: gather candidates, adjacent LCP, per-depth segment bitmaps.  Rows >= R act as terminators.
    const int row_words = (R >> 6) + 1;
    for (int base = wave * 64; base < row_words * 64; base += kThreads) {
        const int r = base + lane;
        // my row, and for lane 0 also the row before it (every other lane finds that one in its neighbour's
        // registers): both suffix-array entries are requested first, then both rows' tokens, 16 bytes a read
        const bool need_prev = lane == 0 && r > 0 && r < R;
        uint32_t start = 0, pstart = 0;
        if (r < R) start = load_sa<SaT>(p.sa, p.n_tokens, kept_entry(r));
        if (need_prev) pstart = load_sa<SaT>(p.sa, p.n_tokens, kept_entry(r - 1));
        if (r < R) rowpos[r] = start;
        int32_t tok[REST_MAX_CONT_LEN], ptok[REST_MAX_CONT_LEN];
        int len, plen0;
        load_row_at<REST_MAX_CONT_LEN, TokT>(p, start, r < R, n_star, tok, len);
        load_row_at<REST_MAX_CONT_LEN, TokT>(p, pstart, need_prev, n_star, ptok, plen0);
        int plen = __shfl_up(len, 1, 64);
        if (need_prev) plen = plen0;
        int l = 0;
        bool run = true;
#pragma unroll
        for (int j = 0; j < REST_MAX_CONT_LEN; j++) {
            if (j < m) {
                int32_t prev = __shfl_up(tok[j], 1, 64);
                if (need_prev) prev = ptok[j];
                run = run && j < len && j < plen && prev == tok[j];
                l += run ? 1 : 0;
            }
        }
        if (r == 0) l = 0;
        if (r < R) { lcp[r] = (uint8_t)l; rlen[r] = (uint8_t)len; }
        {
            const uint64_t cut = __ballot(r < R && len < m);
            if (lane == 0) shortbm[base >> 6] = cut;
        }
        for (int d = 1; d <= m; d++) {
            const uint64_t bits = __ballot(r >= R || l < d);
            if (lane == 0) seg[(d - 1) * words + (base >> 6)] = bits;
        }
    }
    __syncthreads();

    // ---- B1b: per depth, where the next segment starts after each word (one wavefront per depth, words 64 at a
    // time from the top; the terminator bits guarantee a set bit in the last word)
    for (int d = wave; d < m; d += kWavesPerWG) {
        const uint64_t* bm = seg + d * words;
        int32_t carry = row_words * 64;                        // nothing after the last word
        for (int base = ((row_words - 1) / 64) * 64; base >= 0; base -= 64) {
            const int wi = base + lane;
            const uint64_t x = wi < row_words ? bm[wi] : 0ull;
            const uint64_t nz = __ballot(x != 0ull);
            const int first_here = x ? wi * 64 + __builtin_ctzll(x) : 0;
            const uint64_t above = lane < 63 ? nz & (~0ull << (lane + 1)) : 0ull;
            const int src = above ? __builtin_ctzll(above) : 0;
            const int from_lane = __shfl(first_here, src, 64);
            if (wi < row_words) after[d * words + wi] = above ? from_lane : carry;
            if (nz) carry = __shfl(first_here, __builtin_ctzll(nz), 64);
        }
    }
    __syncthreads();

    // ---- B2: weight histogram over all Trie nodes (node (d, r): segment start at depth d with len >= d)
    const int items = m * row_words;   // one item = (depth, 64-row word)
    // eight threads per item, each with eight of its rows; weight-1 nodes are by far the most frequent and are
    // summed over the wavefront before they touch the histogram
    for (int u0 = wave * 64; u0 < items * 8; u0 += kThreads) {
        const int u = u0 + lane;
        uint32_t n_ones = 0;
        if (u < items * 8) {
            const int it = u >> 3, d = it / row_words + 1, wi = it % row_words;
            const uint64_t mine = 0xffull << (8 * (u & 7));
            const Item x = classify(seg, after, shortbm, rlen, words, row_words, d, wi, R);
            n_ones = (uint32_t)popc64(x.ones & mine);
            for (uint64_t rest = x.big & mine; rest; rest &= rest - 1)
                atomicAdd(&hist[bit_weight(x, wi, __builtin_ctzll(rest))], 1u);
        }
        for (int off = 32; off > 0; off >>= 1) n_ones += __shfl_xor(n_ones, off, 64);
        if (lane == 0 && n_ones) atomicAdd(&hist[1], n_ones);
    }
    __syncthreads();

    // ---- B3: boundary weight w*: the largest w with #(weight >= w) >= c (or 1 if the Trie has < c nodes)
    {
        const int per = (p.K + kThreads) / kThreads;           // bins per thread, covering 0..K
        const int b0 = tid * per;
        uint32_t own = 0;
        for (int i = 0; i < per; i++) own += (b0 + i <= p.K) ? hist[b0 + i] : 0;
        // suffix sums over threads: inclusive scan from the top
        uint32_t x = own;
        for (int off = 1; off < 64; off <<= 1) {
            uint32_t y = __shfl_down(x, off, 64);
            if (lane + off < 64) x += y;
        }
        if (lane == 0) part[wave] = x;
        __syncthreads();
        uint32_t above_waves = 0;
        for (int w = wave + 1; w < kWavesPerWG; w++) above_waves += part[w];
        const uint32_t incl = x + above_waves;        // nodes with weight bin >= b0
        const uint32_t excl = incl - own;             // nodes with weight bin >= b0 + per
        if (tid == 0) { s_misc[0] = 1; s_misc[1] = 0; s_misc[5] = (int32_t)incl; }
        __syncthreads();
        if (excl < (uint32_t)c && incl >= (uint32_t)c) {
            uint32_t run_above = excl;
            for (int i = per - 1; i >= 0; i--) {
                const int w = b0 + i;
                const uint32_t hw = w <= p.K ? hist[w] : 0;
                if (run_above + hw >= (uint32_t)c) { s_misc[0] = w; s_misc[1] = (int32_t)run_above; break; }
                run_above += hw;
            }
        }
        __syncthreads();
    }
    const int total_nodes = s_misc[5];
    const bool take_all = total_nodes <= c;
    const int w_star = take_all ? 0 : s_misc[0];          // weight > w_star: always kept
    const int need_w = take_all ? 0 : c - s_misc[1];      // nodes of weight w_star still to take

    // ---- B4: inside weight w*, per-depth counts -> boundary depth d*
    uint32_t* dcount = part + 64;      // [m + 1]
    if (tid <= m) dcount[tid] = 0;
    __syncthreads();
    if (!take_all) {
        for (int u = tid; u < items * 8; u += kThreads) {
            const int it = u >> 3, d = it / row_words + 1, wi = it % row_words;
            const uint64_t mine = 0xffull << (8 * (u & 7));
            const Item x = classify(seg, after, shortbm, rlen, words, row_words, d, wi, R);
            uint32_t n = 0;
            if (w_star == 1) {
                n = (uint32_t)popc64(x.ones & mine);
            } else {
                for (uint64_t rest = x.big & mine; rest; rest &= rest - 1)
                    n += bit_weight(x, wi, __builtin_ctzll(rest)) == w_star;
            }
            if (n) atomicAdd(&dcount[d], n);
        }
    }
    __syncthreads();
    if (tid == 0) {
        int d_star = m + 1, need_d = 0, acc = 0;
        if (!take_all) {
            for (int d = 1; d <= m; d++) {
                if (acc + (int)dcount[d] >= need_w) { d_star = d; need_d = need_w - acc; break; }
                acc += (int)dcount[d];
            }
        }
        s_misc[2] = d_star;
        s_misc[3] = need_d;
        s_misc[4] = 0;   // selection cursor
    }
    __syncthreads();
    const int d_star = s_misc[2], need_d = s_misc[3];

    // ---- B5: inside (w*, d*), rank by row: per-word counts and their exclusive prefix (one wavefront)
    uint32_t* wpre = part + 128;       // [row_words]
    if (!take_all && d_star <= m) {
        for (int wi = tid; wi < row_words; wi += kThreads) {
            const Item x = classify(seg, after, shortbm, rlen, words, row_words, d_star, wi, R);
            uint32_t n = 0;
            if (w_star == 1) {
                n = (uint32_t)popc64(x.ones);
            } else {
                for (uint64_t rest = x.big; rest; rest &= rest - 1) n += bit_weight(x, wi, __builtin_ctzll(rest)) == w_star;
            }
            wpre[wi] = n;
        }
        __syncthreads();
        if (wave == 0) {
            uint32_t carry = 0;
            for (int base = 0; base < row_words; base += 64) {
                const int wi = base + lane;
                const uint32_t v = wi < row_words ? wpre[wi] : 0;
                uint32_t x = v;
                for (int off = 1; off < 64; off <<= 1) {
                    uint32_t y = __shfl_up(x, off, 64);
                    if (lane >= off) x += y;
                }
                if (wi < row_words) wpre[wi] = carry + x - v;
                carry += __shfl(x, 63, 64);
            }
        }
    }
    __syncthreads();

    // ---- B6: select
    // eight threads per item, each with eight of its rows; the kept nodes of a thread take consecutive free slots
    // (the slots are ordered afterwards)
    for (int u = tid; u < items * 8; u += kThreads) {
        const int it = u >> 3, d = it / row_words + 1, wi = it % row_words;
        const uint64_t mine = 0xffull << (8 * (u & 7));
        const Item x = classify(seg, after, shortbm, rlen, words, row_words, d, wi, R);
        // weight-1 nodes are kept only if everything is, or if the boundary weight is 1 and the depth allows it
        const bool ones_matter = take_all || (w_star == 1 && d <= d_star);
        uint64_t keep = (x.big | (ones_matter ? x.ones : 0ull)) & mine;
        if (!take_all) {
            // drop what is too light; at the boundary depth, nodes of the boundary weight are taken in row order
            const bool ranked = d == d_star;
            int rank = 0;
            if (ranked) {
                rank = (int)wpre[wi];
                const uint64_t below = x.node & ~(~0ull << (8 * (u & 7)));
                if (w_star == 1) {
                    rank += popc64(x.ones & below);
                } else {
                    for (uint64_t rest = x.big & below; rest; rest &= rest - 1)
                        rank += bit_weight(x, wi, __builtin_ctzll(rest)) == w_star;
                }
            }
            for (uint64_t rest = keep; rest; rest &= rest - 1) {
                const int b = __builtin_ctzll(rest);
                const int w = ((x.ones >> b) & 1ull) ? 1 : bit_weight(x, wi, b);
                bool ok = w > w_star || (w == w_star && d < d_star);
                if (ranked && w == w_star) ok = rank++ < need_d;
                if (!ok) keep &= ~(1ull << b);
            }
        }
        if (keep) {
            int idx = atomicAdd(&s_misc[4], popc64(keep));
            for (; keep; keep &= keep - 1, idx++) {
                const int b = __builtin_ctzll(keep);
                if (idx < c) {
                    sel_key[idx] = ((uint32_t)d << 16) | (uint32_t)(wi * 64 + b);
                    sel_wgt[idx] = ((x.ones >> b) & 1ull) ? 1u : (uint32_t)bit_weight(x, wi, b);
                }
            }
        }
    }
    __syncthreads();
    int T = s_misc[4];
    T = T > c ? c : T;

    // ---- B7: breadth-first order = ascending (depth, row): rank by counting, four threads per node
    {
        const int x = tid >> 2, part = tid & 3;
        int rank = 0;
        if (x < T) {
            const uint32_t k = sel_key[x];
#pragma unroll 4
            for (int j = part; j < T; j += 4) rank += sel_key[j] < k ? 1 : 0;
        }
        rank += __shfl_xor(rank, 1, 64);
        rank += __shfl_xor(rank, 2, 64);
        if (x < T && part == 0) {
            srt_key[rank] = sel_key[x];
            srt_wgt[rank] = sel_wgt[x];
        }
    }
    __syncthreads();
    // Mask rows and parents, a wavefront per node x, lanes = the 64 slots of a mask word: node a is on the root path
    // of x iff depth(a) <= depth(x) and row(a) <= row(x) < row(a) + weight(a) (a node's rows are consecutive), so a
    // mask word is a ballot; slots are in (depth, row) order, so the parent is the highest slot on the path below x.
    for (int x = wave; x < T; x += kWavesPerWG) {
        const uint32_t kx = srt_key[x];
        const int dx = (int)(kx >> 16), rx = (int)(kx & 0xffff);
        int par = -1;
        for (int k = 0; k < p.mask_words; k++) {
            const int a = 64 * k + lane;
            bool on_path = false;
            if (a < T) {
                const uint32_t ka = srt_key[a];
                const int da = (int)(ka >> 16), ra = (int)(ka & 0xffff);
                on_path = da <= dx && ra <= rx && rx < ra + (int)srt_wgt[a];
            }
            const uint64_t word = __ballot(on_path);
            const uint64_t above = (x >> 6) == k ? word & ~(1ull << (x & 63)) : word;
            if (above) par = 64 * k + 63 - __builtin_clzll(above);
            if (lane == 0) o_mask[(int64_t)x * p.mask_words + k] = word;
        }
        if (lane == 0) {
            o_tok[x] = load_tok<TokT>(p.corpus, p.n_tokens, (uint64_t)rowpos[rx] + n_star + (dx - 1));
            o_par[x] = par;
            o_pos[x] = dx;
            o_wgt[x] = (int32_t)srt_wgt[x];
        }
    }
    for (int i = T + tid; i < c; i += kThreads) {
        o_tok[i] = -1; o_par[i] = -1; o_pos[i] = 0; o_wgt[i] = 0;
        for (int w = 0; w < p.mask_words; w++) o_mask[(int64_t)i * p.mask_words + w] = 0;
    }
    if (tid == 0) {
        p.out.n_nodes[b] = T;
        p.out.matched_len[b] = n_star;
        p.out.match_count[b] = (int64_t)(hi - lo);
    }
}

// Fills the sampled-key table: key k = first 16 tokens (-1 past the end of the stream) of the suffix of rank
// rest_top_rank(n, top_count, k); words that belong to no key are 0.
template <typename TokT, typename SaT>
__global__ void top_table_kernel(const void* corpus, const void* sa, uint64_t n, int32_t top_count, int32_t* tab) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= table_words(top_count)) return;
    int k, j = -1;                                   // j = -1: the rank itself
    if (i < kCoarse) { j = i / 64; k = 16 * (i % 64) + 15; }
    else if (i < kTabKeys) k = i - kCoarse;
    else { const int w = i - kTabKeys; k = 16 * (w / 256) + w % 16; j = (w % 256) / 16; }
    int32_t v = 0;
    if (k < top_count) {
        const uint32_t rank = (uint32_t)rest_top_rank(n, top_count, k);
        v = j < 0 ? (int32_t)rank : load_tok<TokT>(corpus, n, (uint64_t)load_sa<SaT>(sa, n, rank) + j);
    }
    tab[i] = v;
}

bool params_ok(const rest_retrieve_params* q) {
    if (!q) return false;
    if (q->n_max < 1 || q->n_max > REST_MAX_SUFFIX_LEN || q->n_min < 1 || q->n_min > q->n_max) return false;
    if (q->max_matches < 1 || q->max_matches > REST_MAX_MATCHES) return false;
    if (q->cont_len < 1 || q->cont_len > REST_MAX_CONT_LEN) return false;
    if (q->max_nodes < 1 || q->max_nodes > REST_MAX_NODES) return false;
    if (q->random_seqs < 0 || q->random_seqs > 64) return false;
    if (q->strided != 0 && q->strided != 1) return false;
    return true;
}

size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

template <typename TokT, typename SaT>
rest_status launch(const RetrieveParams& p, int B, size_t lds_bytes, hipStream_t stream) {
    auto kern = retrieve_kernel<TokT, SaT>;
    // raise the kernel's dynamic-LDS limit once per (instantiation, device) and only when a call needs more
    static size_t granted[64] = {0};
    static std::mutex granted_lock;                 // host threads may call at once
    int dev = 0;
    REST_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return REST_UNSUPPORTED;
    {
        std::lock_guard<std::mutex> hold(granted_lock);
        if (lds_bytes > granted[dev]) {
            REST_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));
            granted[dev] = lds_bytes;
        }
    }
    hipLaunchKernelGGL(kern, dim3(B), dim3(kThreads), lds_bytes, stream, p);
    REST_HIP_TRY(hipGetLastError());
    REST_BOUNDS_EPILOGUE(stream);
    return REST_OK;
}

}  // namespace

rest_status rest_internal_make_top_table(rest_index* idx, hipStream_t stream) {
    int tc = (int)(idx->n_tokens / 64 < (uint64_t)kTopMax ? idx->n_tokens / 64 : (uint64_t)kTopMax);
    idx->top_count = tc;
    // always allocate so the pointer is valid
    if (hipMalloc((void**)&idx->d_top_keys, (size_t)table_words(tc) * sizeof(int32_t)) != hipSuccess) {
        (void)hipGetLastError();
        idx->d_top_keys = nullptr;
        return REST_OUT_OF_MEMORY;
    }
    if (tc > 0) {
        const int total = table_words(tc), blocks = (total + 255) / 256;
        if (idx->token_bytes == 2 && idx->sa_bytes == 4)
            hipLaunchKernelGGL((top_table_kernel<uint16_t, int32_t>), dim3(blocks), dim3(256), 0, stream, idx->d_corpus, idx->d_sa, idx->n_tokens, tc, idx->d_top_keys);
        else if (idx->token_bytes == 2)
            hipLaunchKernelGGL((top_table_kernel<uint16_t, int64_t>), dim3(blocks), dim3(256), 0, stream, idx->d_corpus, idx->d_sa, idx->n_tokens, tc, idx->d_top_keys);
        else if (idx->sa_bytes == 4)
            hipLaunchKernelGGL((top_table_kernel<int32_t, int32_t>), dim3(blocks), dim3(256), 0, stream, idx->d_corpus, idx->d_sa, idx->n_tokens, tc, idx->d_top_keys);
        else
            hipLaunchKernelGGL((top_table_kernel<int32_t, int64_t>), dim3(blocks), dim3(256), 0, stream, idx->d_corpus, idx->d_sa, idx->n_tokens, tc, idx->d_top_keys);
        REST_HIP_TRY(hipGetLastError());
    }
    REST_HIP_TRY(hipStreamSynchronize(stream));
    REST_BOUNDS_EPILOGUE(stream);
    return REST_OK;
}

extern "C" __attribute__((visibility("default"))) size_t rest_retrieve_workspace_bytes(int32_t B, const rest_retrieve_params* params) {
    // every intermediate lives in LDS; the workspace argument is kept in the ABI for forward compatibility
    (void)B;
    (void)params;
    return 0;
}

extern "C" __attribute__((visibility("default"))) rest_status rest_retrieve(const rest_index* index, const int32_t* d_contexts, const int32_t* d_ctx_len,
                                     int32_t B, int32_t ctx_stride, const rest_retrieve_params* q,
                                     const rest_tree* out, void* d_workspace, size_t workspace_bytes, void* stream_) {
    (void)d_workspace;
    (void)workspace_bytes;
    if (!index || !params_ok(q) || !out) return REST_INVALID_ARG;
    if (B < 0 || ctx_stride < 0) return REST_INVALID_ARG;
    // a depth-limited index orders positions by sort_depth tokens only; the search reads n_max of them and the
    // adjacent-row comparison cont_len more
    if (index->sort_depth > 0 && q->n_max + q->cont_len > index->sort_depth) return REST_UNSUPPORTED;
    if (B == 0) return REST_OK;
    if (!d_contexts || !d_ctx_len) return REST_INVALID_ARG;
    if (!out->draft_tokens || !out->parent_idx || !out->pos_ids || !out->node_weight || !out->tree_mask ||
        !out->n_nodes || !out->matched_len || !out->match_count)
        return REST_INVALID_ARG;

    RetrieveParams p;
    p.corpus = index->d_corpus;
    p.sa = index->d_sa;
    p.top_keys = index->d_top_keys;
    p.n_tokens = index->n_tokens;
    p.top_count = index->top_count;
    p.contexts = d_contexts;
    p.ctx_len = d_ctx_len;
    p.ctx_stride = ctx_stride;
    p.n_max = q->n_max; p.n_min = q->n_min; p.K = q->max_matches; p.m = q->cont_len; p.c = q->max_nodes;
    p.mask_words = (q->max_nodes + 63) / 64;
    p.random_seqs = q->random_seqs;
    p.seed = q->seed;
    p.strided = q->strided;
    p.out = *out;
    p.words = p.K / 64 + 1;
    size_t off = 0;
    p.off_seg = (int32_t)off;  off = align16(off + (size_t)p.m * p.words * 8);
    p.off_lcp = (int32_t)off;  off = align16(off + (size_t)p.K);
    p.off_len = (int32_t)off;  off = align16(off + (size_t)p.K);
    p.off_hist = (int32_t)off; off = align16(off + (size_t)(p.K + 1) * 4);
    p.off_part = (int32_t)off; off = align16(off + (size_t)(128 + p.words + 64) * 4);
    p.off_sel = (int32_t)off;  off = align16(off + (size_t)REST_MAX_NODES * 5 * 4);
    p.off_pos = (int32_t)off;  off = align16(off + (size_t)p.K * 4);
    p.off_after = (int32_t)off; off = align16(off + (size_t)p.m * p.words * 4);
    p.off_short = (int32_t)off; off = align16(off + (size_t)p.words * 8);
    p.off_misc = (int32_t)off;
    size_t lds_bytes = off;
    const size_t top_bytes = (size_t)table_words(index->top_count) * 4;
    if (top_bytes > lds_bytes) lds_bytes = top_bytes;
    if ((size_t)kFewBytes > lds_bytes) lds_bytes = kFewBytes;
    if (lds_bytes > 150 * 1024) return REST_UNSUPPORTED;

    hipStream_t stream = (hipStream_t)stream_;
    if (index->token_bytes == 2 && index->sa_bytes == 4) return launch<uint16_t, int32_t>(p, B, lds_bytes, stream);
    if (index->token_bytes == 2) return launch<uint16_t, int64_t>(p, B, lds_bytes, stream);
    if (index->sa_bytes == 4) return launch<int32_t, int32_t>(p, B, lds_bytes, stream);
    return launch<int32_t, int64_t>(p, B, lds_bytes, stream);
}
