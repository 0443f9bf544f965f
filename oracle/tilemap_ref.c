/* Oracle (test infrastructure only): the tile map of paper section 3.2.1 as
 * the literal double loop over (query, key) pairs, in plain C, for sequence
 * lengths where the NumPy version is too slow.  Shares nothing with the HIP
 * library.  Pinned against oracle/tilemap.py and closed forms in
 * tests/test_oracle_mask.py.
 *
 *   vis(q,k) = sample[q]==sample[k] &&
 *              ((causal[q] && k<=q && bit modality[k] of attend[q] &&
 *                (window[q]==0 || modality[q]!=modality[k] || q-k<window[q])) ||
 *               (span[q]!=0 && span[q]==span[k]))
 *   cnt[i][j] = number of visible pairs in q-tile i x k-tile j
 *   cls = 0 EMPTY (cnt==0), 1 FULL (cnt==tq*tk), 2 PARTIAL
 *   W[i] = sum_j cnt[i][j]
 */
#include <stdint.h>

int tilemap_ref(const int64_t* sample, const int64_t* span, const int64_t* causal,
                const int64_t* modality, const int64_t* attend, const int64_t* window,
                int64_t S, int32_t tq, int32_t tk,
                uint8_t* cls, uint32_t* cnt, uint64_t* W)
{
    if (S % tq || S % tk) return -1;
    int64_t nq = S / tq, nk = S / tk;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < nq; ++i) {
        uint64_t w = 0;
        for (int64_t j = 0; j < nk; ++j) {
            uint32_t c = 0;
            for (int64_t q = i * tq; q < (i + 1) * tq; ++q)
                for (int64_t k = j * tk; k < (j + 1) * tk; ++k) {
                    int same_sample = sample[q] == sample[k];
                    int back = causal[q] && k <= q && ((attend[q] >> modality[k]) & 1);
                    if (window[q] != 0 && modality[q] == modality[k] && q - k >= window[q]) back = 0;
                    int same_span = span[q] != 0 && span[q] == span[k];
                    c += (uint32_t)(same_sample && (back || same_span));
                }
            cnt[i * nk + j] = c;
            cls[i * nk + j] = c == 0 ? 0 : (c == (uint32_t)tq * (uint32_t)tk ? 1 : 2);
            w += c;
        }
        W[i] = w;
    }
    return 0;
}
