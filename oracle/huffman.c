/*
 * CPU oracle (test infrastructure): Huffman table construction.
 * T.81 Annex C (canonical codes from BITS) and Annex K.2 (code lengths from
 * symbol counts, limited to 16 bits, no all-ones code).
 */
#include "oracle.h"
#include <string.h>

/* Annex C: codes of one length are consecutive integers; moving to the next
 * length appends a zero bit.                                               */
int oracle_huff_codes(const uint8_t bits[17], uint16_t code[256], uint8_t size[256])
{
    int n = 0;
    uint32_t next = 0;
    for (int len = 1; len <= 16; len++) {
        for (int i = 0; i < bits[len]; i++) {
            if (n >= 256) return ORACLE_E_CORRUPT;
            if (next >= (1u << len)) return ORACLE_E_CORRUPT; /* over-subscribed */
            code[n] = (uint16_t)next;
            size[n] = (uint8_t)len;
            next++;
            n++;
        }
        next <<= 1;
    }
    return n;
}

/* Annex K.2.  A 257th pseudo-symbol with count 1 takes the longest code, so
 * the all-ones code word stays unused.  Lengths come from repeatedly joining
 * the two rarest groups; every member of a joined group gets one bit longer. */
int oracle_huff_from_freq(const int64_t freq_in[256], uint8_t bits[17], uint8_t huffval[256])
{
    int64_t freq[257];
    int group[257];    /* group id of each symbol, -1 = not coded */
    int length[257];
    for (int i = 0; i < 256; i++) freq[i] = freq_in[i] > 0 ? freq_in[i] : 0;
    freq[256] = 1;
    int64_t gfreq[257];
    int galive[257];
    for (int i = 0; i < 257; i++) {
        group[i] = freq[i] > 0 ? i : -1;
        gfreq[i] = freq[i];
        galive[i] = freq[i] > 0;
        length[i] = 0;
    }
    for (;;) {
        /* rarest and second rarest live groups; ties go to the larger id */
        int a = -1, b = -1;
        for (int g = 0; g < 257; g++) {
            if (!galive[g]) continue;
            if (a < 0 || gfreq[g] <= gfreq[a]) a = g;
        }
        for (int g = 0; g < 257; g++) {
            if (!galive[g] || g == a) continue;
            if (b < 0 || gfreq[g] <= gfreq[b]) b = g;
        }
        if (b < 0) break;
        for (int s = 0; s < 257; s++)
            if (group[s] == a || group[s] == b) {
                length[s]++;
                group[s] = a;
            }
        gfreq[a] += gfreq[b];
        galive[b] = 0;
    }
    int count[64];
    memset(count, 0, sizeof count);
    for (int s = 0; s < 257; s++)
        if (freq[s] > 0) {
            if (length[s] >= 64) return ORACLE_E_ARG;
            count[length[s]]++;
        }
    /* limit to 16 bits: take a pair from length i, give one member the
     * prefix (length i-1), and split a shorter code word to host the other. */
    for (int i = 63; i > 16; i--)
        while (count[i] > 0) {
            int j = i - 2;
            while (j > 0 && count[j] == 0) j--;
            if (j <= 0) return ORACLE_E_ARG;
            count[i] -= 2;
            count[i - 1] += 1;
            count[j + 1] += 2;
            count[j] -= 1;
        }
    /* drop the reserved pseudo-symbol from the longest length in use */
    int longest = 16;
    while (longest > 0 && count[longest] == 0) longest--;
    if (longest == 0) return ORACLE_E_ARG;
    count[longest]--;
    bits[0] = 0;
    for (int l = 1; l <= 16; l++) bits[l] = (uint8_t)count[l];
    /* symbols ordered by their (pre-limit) length, then by value */
    int n = 0;
    for (int l = 1; l < 64; l++)
        for (int s = 0; s < 256; s++)
            if (freq[s] > 0 && length[s] == l) huffval[n++] = (uint8_t)s;
    return n;
}
