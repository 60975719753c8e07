/* Drives the C part of the CPU oracle over many small, irregular inputs.  Built by the test suite with
 * -fsanitize=address,undefined: any out-of-bounds access, overflow or leak in the oracle ends the run with a report.
 * The results themselves are checked elsewhere (the oracle's pins); here only a few cheap invariants are. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_suffix_array(const void *corpus, uint64_t n, int token_bytes, int64_t *sa_out);
int64_t oracle_check_suffix_array(const void *corpus, uint64_t n, int token_bytes, const void *sa, int sa_bytes);
int oracle_retrieve(const void *corpus, uint64_t n_tokens, int token_bytes, const int32_t *s, int32_t t,
                    int32_t n_max, int32_t n_min, int64_t K, int32_t m, int32_t mode,
                    int32_t *matched_len, int64_t *match_count, int64_t *n_rows,
                    int64_t *row_pos, int32_t *rows, int32_t *row_len);
int oracle_select_drafts(const int32_t *rows, const int32_t *row_len, const int64_t *order, int64_t R, int32_t m,
                         int32_t c, int32_t words, int32_t *n_nodes, int32_t *tok, int32_t *par, int32_t *pos,
                         int32_t *wgt, uint64_t *mask, int64_t *total_nodes);
int oracle_accept(const int32_t *ids, const int32_t *draft_tokens, const int32_t *parent_idx, int32_t n_nodes, int32_t m,
                  int32_t *accept_len, int32_t *accept_path, int32_t *next_token);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(uint32_t n) {
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (uint32_t)((state >> 33) % (n ? n : 1));
}
#define CHECK(x) do { if (!(x)) { fprintf(stderr, "check failed: %s (line %d)\n", #x, __LINE__); return 1; } } while (0)

int main(void) {
    for (int iter = 0; iter < 400; iter++) {
        const int tb = rnd(2) ? 4 : 2;
        const uint64_t n = 1 + rnd(iter < 50 ? 4 : 600);
        const uint32_t vocab = 1 + rnd(4);
        void *corpus = malloc(n * tb);
        for (uint64_t i = 0; i < n; i++) {
            if (tb == 4) ((int32_t *)corpus)[i] = (int32_t)rnd(vocab); else ((uint16_t *)corpus)[i] = (uint16_t)rnd(vocab);
        }
        int64_t *sa = malloc(n * sizeof *sa);
        CHECK(oracle_suffix_array(corpus, n, tb, sa) == 0);
        CHECK(oracle_check_suffix_array(corpus, n, tb, sa, 8) == -1);
        if (n > 1) { int64_t x = sa[0]; sa[0] = sa[1]; sa[1] = x; CHECK(oracle_check_suffix_array(corpus, n, tb, sa, 8) >= 0); }

        const int32_t t = (int32_t)rnd(24), n_max = 1 + (int32_t)rnd(16), n_min = 1 + (int32_t)rnd((uint32_t)n_max);
        const int64_t K = rnd(3) ? (int64_t)rnd(40) : 0;
        const int32_t m = (int32_t)rnd(12);
        int32_t *s = malloc((t ? t : 1) * sizeof *s);
        for (int32_t i = 0; i < t; i++) s[i] = (int32_t)rnd(vocab + 1);
        int64_t *row_pos = malloc((K + 1) * sizeof *row_pos);
        int32_t *rows = malloc((K + 1) * (m ? m : 1) * sizeof *rows), *row_len = malloc((K + 1) * sizeof *row_len);
        int32_t ml[2];
        int64_t mc[2], nr[2];
        for (int mode = 0; mode < 2; mode++) {
            CHECK(oracle_retrieve(corpus, n, tb, s, t, n_max, n_min, K, m, mode, &ml[mode], &mc[mode], &nr[mode], row_pos, rows,
                                  row_len) == 0);
            CHECK(nr[mode] <= K && nr[mode] <= mc[mode]);
        }
        CHECK(ml[0] == ml[1] && mc[0] == mc[1] && nr[0] == nr[1]);

        const int64_t R = nr[1];
        const int32_t c = 1 + (int32_t)rnd(70), words = (c + 63) / 64;
        int32_t *tok = malloc(c * sizeof *tok), *par = malloc(c * sizeof *par), *pos = malloc(c * sizeof *pos), *wgt = malloc(c * sizeof *wgt);
        uint64_t *mask = malloc((size_t)c * words * sizeof *mask);
        int32_t nn = 0;
        int64_t total = 0;
        if (m > 0) {
            CHECK(oracle_select_drafts(rows, row_len, NULL, R, m, c, words, &nn, tok, par, pos, wgt, mask, &total) == 0);
            CHECK(nn <= c && nn <= total);
            int32_t *ids = malloc((1 + c) * sizeof *ids);
            for (int32_t i = 0; i <= c; i++) ids[i] = (int32_t)rnd(vocab + 1);
            const int32_t cap = 1 + (int32_t)rnd(12);
            int32_t alen = 0, nxt = 0, *path = malloc(cap * sizeof *path);
            CHECK(oracle_accept(ids, tok, par, nn, cap, &alen, path, &nxt) == 0);
            CHECK(alen >= 0 && alen <= cap);
            free(path); free(ids);
        }
        free(mask); free(wgt); free(pos); free(par); free(tok);
        free(row_len); free(rows); free(row_pos); free(s); free(sa); free(corpus);
    }
    printf("oracle sanitizer drive: ok\n");
    return 0;
}
