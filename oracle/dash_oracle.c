/*
 * dash_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded CPU garbler / evaluator for arithmetic garbled
 * circuits over CRT residues, written from the Dash paper (arXiv 2302.06361).
 * It exists to check the GPU library; nothing in the product path may call it.
 * It shares no code, header, table or constant generator with the GPU library.
 *
 * Every function cites the passage of the paper it follows.  Where the paper is
 * silent the reading that is implemented is stated next to the code.
 *
 * Layouts used by this file (host memory, all labels one byte per digit):
 *   label tensor of modulus m  : [elem][lambda_m]              (compact)
 *   ciphertext segment of a gate batch p -> q over E elements :
 *                                [elem][row 0..p-1][pitch_q],  pitch_q = 4*ceil(lambda_q/4),
 *                                pad bytes zero
 *   a layer's table buffer     : its segments in slot order; segment s starts at
 *                                E * (sum of rows*pitch of the segments before s)
 *
 * Pins (tests/, CPU only): FIPS-197 vectors and the openssl CLI for AES, Python
 * big integers for compress / decompress / CRT, brute force over all inputs of every
 * gate for small moduli, [X >= P/2] for every X on small CRT bases, the paper's
 * scaling table for Z_6, ceil(x/2) for every x on small bases, and the decoded
 * result of whole networks against plain integer evaluation.
 * The label and ciphertext BYTES depend on readings the paper leaves open (hash,
 * tweak, PRG): those bytes are "parity unpinned" by the paper; they are pinned only
 * through the invariants above.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef unsigned __int128 u128;
typedef uint8_t u8;
typedef uint64_t u64;

#define MAXK 16
#define MAXN 16
#define MAXLAM 128

/* ------------------------------------------------------------------------- */
/* AES-128 encryption, byte oriented, straight from FIPS-197.                */
/* (Sec. "Garbled Circuit Optimizations": fixed-key AES as the permutation.) */
/* ------------------------------------------------------------------------- */

static u8 SBOX[256];
static int sbox_ready = 0;

static u8 gf_mul(u8 a, u8 b) {           /* multiplication in GF(2^8) mod x^8+x^4+x^3+x+1 */
    u8 r = 0;
    while (b) {
        if (b & 1) r ^= a;
        a = (u8)((a << 1) ^ ((a & 0x80) ? 0x1b : 0));
        b >>= 1;
    }
    return r;
}

static void sbox_init(void) {
    /* FIPS-197 5.1.1: multiplicative inverse, then the affine map with constant 0x63 */
    for (int x = 0; x < 256; x++) {
        u8 inv = 0;
        if (x) for (int y = 1; y < 256; y++) if (gf_mul((u8)x, (u8)y) == 1) { inv = (u8)y; break; }
        u8 s = 0;
        for (int i = 0; i < 8; i++) {
            int bit = ((inv >> i) ^ (inv >> ((i + 4) & 7)) ^ (inv >> ((i + 5) & 7)) ^
                       (inv >> ((i + 6) & 7)) ^ (inv >> ((i + 7) & 7)) ^ (0x63 >> i)) & 1;
            s |= (u8)(bit << i);
        }
        SBOX[x] = s;
    }
    sbox_ready = 1;
}

/* FIPS-197 5.2: key expansion, 11 round keys of 16 bytes */
static void aes_expand(const u8 key[16], u8 rk[176]) {
    if (!sbox_ready) sbox_init();
    memcpy(rk, key, 16);
    u8 rcon = 1;
    for (int w = 4; w < 44; w++) {
        u8 t[4];
        memcpy(t, rk + 4 * (w - 1), 4);
        if (w % 4 == 0) {
            u8 t0 = t[0];
            t[0] = (u8)(SBOX[t[1]] ^ rcon); t[1] = SBOX[t[2]]; t[2] = SBOX[t[3]]; t[3] = SBOX[t0];
            rcon = gf_mul(rcon, 2);
        }
        for (int b = 0; b < 4; b++) rk[4 * w + b] = (u8)(rk[4 * (w - 4) + b] ^ t[b]);
    }
}

/* FIPS-197 5.1: cipher.  State byte s[r][c] = in[r + 4c]. */
static void aes_encrypt(const u8 rk[176], const u8 in[16], u8 out[16]) {
    u8 s[16], t[16];
    for (int i = 0; i < 16; i++) s[i] = (u8)(in[i] ^ rk[i]);
    for (int round = 1; round <= 10; round++) {
        for (int i = 0; i < 16; i++) s[i] = SBOX[s[i]];                 /* SubBytes */
        for (int c = 0; c < 4; c++)                                     /* ShiftRows */
            for (int r = 0; r < 4; r++) t[r + 4 * c] = s[r + 4 * ((c + r) & 3)];
        if (round < 10) {                                               /* MixColumns */
            for (int c = 0; c < 4; c++) {
                u8 *a = t + 4 * c;
                s[4 * c + 0] = (u8)(gf_mul(a[0], 2) ^ gf_mul(a[1], 3) ^ a[2] ^ a[3]);
                s[4 * c + 1] = (u8)(a[0] ^ gf_mul(a[1], 2) ^ gf_mul(a[2], 3) ^ a[3]);
                s[4 * c + 2] = (u8)(a[0] ^ a[1] ^ gf_mul(a[2], 2) ^ gf_mul(a[3], 3));
                s[4 * c + 3] = (u8)(gf_mul(a[0], 3) ^ a[1] ^ a[2] ^ gf_mul(a[3], 2));
            }
        } else memcpy(s, t, 16);
        for (int i = 0; i < 16; i++) s[i] ^= rk[16 * round + i];        /* AddRoundKey */
    }
    memcpy(out, s, 16);
}

void orc_aes128_encrypt(const u8 key[16], const u8 in[16], u8 out[16]) {
    u8 rk[176];
    aes_expand(key, rk);
    aes_encrypt(rk, in, out);
}

/* 128-bit integer <-> 16 bytes, little endian */
static u128 load128(const u8 b[16]) {
    u128 v = 0;
    for (int i = 15; i >= 0; i--) v = (v << 8) | b[i];
    return v;
}
static void store128(u128 v, u8 b[16]) {
    for (int i = 0; i < 16; i++) { b[i] = (u8)v; v >>= 8; }
}

/* ------------------------------------------------------------------------- */
/* Label length, compress, decompress                                        */
/* ------------------------------------------------------------------------- */

/* Label length for modulus m (Sec. LabelTensors, figure caption: a label must pack
 * into / fill a 128-bit chunk).  rule 0: the smallest lambda with m^lambda >= 2^128
 * (at least 128 bits of entropy); rule 1: the largest lambda with m^lambda <= 2^128
 * (the caption's floor(128 / log2 m)).  Integer arithmetic, no logarithms. */
int orc_lambda(int m, int rule) {
    const u128 limit = (~(u128)0) / (u128)m;     /* v <= limit  <=>  v*m < 2^128 */
    u128 v = 1;
    int lam = 0;
    while (v <= limit) { v *= (u128)m; lam++; }  /* ends with m^lam < 2^128 <= m^(lam+1) */
    /* m^(lam+1) == 2^128 exactly only for m = 2, 4, 16: then both rules give lam+1 */
    if (m == 2 || m == 4 || m == 16) return lam + 1;
    return rule == 0 ? lam + 1 : lam;
}

static int pitch_of(int lam) { return 4 * ((lam + 3) / 4); }

/* compress(l) = (...(l_n q + l_{n-1}) q + ...) q + l_1  (Sec. Implementation), taken
 * mod 2^128 when the label is longer than 128 bits.  L[0] is the paper's l_1. */
static u128 compress(const u8 *L, int lam, int q) {
    u128 acc = 0;
    for (int j = lam - 1; j >= 0; j--) acc = acc * (u128)q + L[j];
    return acc;
}

/* decompress: the base-q digits of a 128-bit number, least significant first; the
 * inverse of compress on its range ("label de-/compression", Sec. LabelTensors). */
static void decompress(u128 h, int q, int lam, u8 *out) {
    for (int j = 0; j < lam; j++) { out[j] = (u8)(h % (u128)q); h /= (u128)q; }
}

void orc_compress(const u8 *L, int lam, int q, u8 out16[16]) { store128(compress(L, lam, q), out16); }
void orc_decompress(const u8 h16[16], int q, int lam, u8 *out) { decompress(load128(h16), q, lam, out); }

/* ------------------------------------------------------------------------- */
/* Context: CRT base, label lengths, offsets, mixed-radix digits             */
/* ------------------------------------------------------------------------- */

typedef struct {
    int k;
    int prime[MAXK];
    int rule;
    u8 rk_fixed[176];          /* fixed public AES key 00 01 .. 0f */
    u8 rk_seed[176];           /* PRG key = the 16-byte seed */
    int n;                     /* mixed-radix digits d_1 (most significant) .. d_n */
    int d[MAXN + 1];           /* 1-based */
    int mj[MAXN + 1];          /* accumulation modulus of digit j: m_1 = d_1, m_j = k*d_j */
    u64 P;                     /* product of the primes */
    u128 M;                    /* product of the digits */
    int lam[256];              /* label length per modulus 2..255 */
    u8 delta[256][MAXLAM];     /* offset label per modulus */
    u8 one0[MAXK][MAXLAM];     /* zero label of the constant-one wire per prime */
} octx;

enum { DOM_DELTA = 0, DOM_INPUT = 1, DOM_GATE = 2, DOM_MASK = 3, DOM_ONE = 4 };

/* PRG (the paper draws labels from a hardware RNG, Sec. Implementation; a seeded
 * counter-based generator replaces it so that any wire can be recomputed alone):
 * block = AES_seed( elem:u64 | slot:u32 | layer:u16 | domain:u8 | modulus:u8 ), little
 * endian; the draw is decompress_m(block). */
static void draw(const octx *c, int domain, int layer, uint32_t slot, u64 elem, int m, u8 *out) {
    u8 blk[16], enc[16];
    for (int i = 0; i < 8; i++) blk[i] = (u8)(elem >> (8 * i));
    for (int i = 0; i < 4; i++) blk[8 + i] = (u8)(slot >> (8 * i));
    blk[12] = (u8)layer; blk[13] = (u8)(layer >> 8);
    blk[14] = (u8)domain; blk[15] = (u8)m;
    aes_encrypt(c->rk_seed, blk, enc);
    decompress(load128(enc), m, c->lam[m], out);
}

/* Hash of a label into Z_q^lambda_q (Sec. Garbled Circuit Optimizations: fixed-key AES
 * as a random permutation; Sec. Implementation: labels are compressed to 128 bits
 * first).  K = compress_p(L); X = K xor tweak; h = AES_fixed(X) xor X;
 * H = decompress_q(h).  tweak = elem:u64 | slot:u32 | layer:u16 | 0:u16. */
/* every ciphertext costs the garbler exactly one hash: a way to count them (per calling thread) */
static __thread unsigned long long hash_calls;
unsigned long long orc_hash_calls(void) { return hash_calls; }
static void hash(const octx *c, const u8 *L, int p, int layer, uint32_t slot, u64 elem, int q, u8 *out) {
    hash_calls++;
    u128 K = compress(L, c->lam[p], p);
    u128 T = (u128)elem | ((u128)slot << 64) | ((u128)(layer & 0xffff) << 96);
    u128 X = K ^ T;
    u8 xb[16], eb[16];
    store128(X, xb);
    aes_encrypt(c->rk_fixed, xb, eb);
    decompress(load128(eb) ^ X, q, c->lam[q], out);
}

/* lam_primes: NULL, or k explicit label lengths (1..128) for the CRT primes in place of the rule
 * (the label length is a parameter of the scheme, Sec. LabelTensors); the accumulation moduli of
 * the sign gadget keep the rule. */
octx *orc_ctx_create(const int *primes, int k, int rule, const int *lam_primes, const u8 seed[16], const int *digits, int n) {
    if (k < 1 || k > MAXK || n < 1 || n > MAXN) return NULL;
    for (int i = 0; lam_primes && i < k; i++) if (lam_primes[i] < 1 || lam_primes[i] > MAXLAM) return NULL;
    octx *c = (octx *)calloc(1, sizeof(octx));
    c->k = k; c->rule = rule; c->n = n;
    c->P = 1;
    for (int i = 0; i < k; i++) { c->prime[i] = primes[i]; c->P *= (u64)primes[i]; }
    c->M = 1;
    for (int j = 1; j <= n; j++) { c->d[j] = digits[j - 1]; c->M *= (u128)digits[j - 1]; }
    /* accumulation moduli (Appendix, Garbled Mixed-Radix Addition): the sum of k digits
     * below d_j plus a carry below k is below k*d_j; the top digit is only needed mod d_1. */
    c->mj[1] = c->d[1];
    for (int j = 2; j <= n; j++) c->mj[j] = k * c->d[j];
    u8 fixed[16];
    for (int i = 0; i < 16; i++) fixed[i] = (u8)i;
    aes_expand(fixed, c->rk_fixed);
    aes_expand(seed, c->rk_seed);
    for (int m = 2; m < 256; m++) {
        c->lam[m] = orc_lambda(m, rule);
        for (int i = 0; lam_primes && i < k; i++) if (primes[i] == m) c->lam[m] = lam_primes[i];
        /* offset label R_m: random, point-and-permute component fixed to 1
         * (Sec. Arithmetic Garbled Circuits).  Component 0 is the colour. */
        draw(c, DOM_DELTA, 0, 0, 0, m, c->delta[m]);
        c->delta[m][0] = 1;
    }
    for (int i = 0; i < k; i++) draw(c, DOM_ONE, 0, 0, 0, c->prime[i], c->one0[i]);
    return c;
}
void orc_ctx_free(octx *c) { free(c); }

int orc_ctx_lambda(const octx *c, int m) { return c->lam[m]; }
void orc_ctx_delta(const octx *c, int m, u8 *out) { memcpy(out, c->delta[m], (size_t)c->lam[m]); }
void orc_ctx_one0(const octx *c, int i, u8 *out) { memcpy(out, c->one0[i], (size_t)c->lam[c->prime[i]]); }
int orc_ctx_mj(const octx *c, int j) { return c->mj[j]; }

void orc_hash(const octx *c, const u8 *L, int p, int layer, uint32_t slot, u64 elem, int q, u8 *out) {
    hash(c, L, p, layer, slot, elem, q, out);
}
void orc_draw(const octx *c, int domain, int layer, uint32_t slot, u64 elem, int m, u8 *out) {
    draw(c, domain, layer, slot, elem, m, out);
}

/* Zero labels of circuit-input wires first_wire .. first_wire+n-1 for prime index i. */
void orc_input_labels(const octx *c, u64 first_wire, long n, int i, u8 *out) {
    int p = c->prime[i], lam = c->lam[p];
    for (long e = 0; e < n; e++) draw(c, DOM_INPUT, 0, 0, first_wire + (u64)e, p, out + e * lam);
}

/* ------------------------------------------------------------------------- */
/* Label arithmetic (Sec. Arithmetic Garbled Circuits: free gates)           */
/* ------------------------------------------------------------------------- */

/* dst = a + c*b  (componentwise mod m); c may be any non-negative int */
static void lab_axpy(u8 *dst, const u8 *a, long c, const u8 *b, int lam, int m) {
    long cm = ((c % m) + m) % m;
    for (int j = 0; j < lam; j++) dst[j] = (u8)(((long)a[j] + cm * (long)b[j]) % m);
}
static void lab_zero(u8 *dst, int lam) { memset(dst, 0, (size_t)lam); }

/* ------------------------------------------------------------------------- */
/* Projection gate (Sec. Arithmetic Garbled Circuits, "Projections for unary */
/* functions"; point-and-permute from Sec. Garbled Circuit Optimizations)    */
/* ------------------------------------------------------------------------- */

/* Garble one gate phi: Z_p -> Z_q on the wire with zero label in0.
 * out0 is the (already chosen) zero label of the output wire.
 * rows[colour(l^a)] = out0 + phi(a)*R_q + H_q(l^a, tweak),  l^a = in0 + a*R_p.
 * rows == NULL: nothing is written (the zero labels of a circuit do not depend on its
 * ciphertexts, so a caller that only needs zero labels skips them). */
static void proj_garble_one(const octx *c, int p, int q, const u8 *in0, const u8 *phi, const u8 *out0,
                            int layer, uint32_t slot, u64 elem, u8 *rows) {
    int lp = c->lam[p], lq = c->lam[q], pitch = pitch_of(lq);
    u8 la[MAXLAM], h[MAXLAM], pay[MAXLAM];
    if (!rows) return;      /* zero labels only: the caller wants no ciphertexts */
    for (int a = 0; a < p; a++) {
        lab_axpy(la, in0, a, c->delta[p], lp, p);
        hash(c, la, p, layer, slot, elem, q, h);
        lab_axpy(pay, out0, phi[a], c->delta[q], lq, q);
        u8 *row = rows + (size_t)la[0] * pitch;
        memset(row, 0, (size_t)pitch);
        for (int j = 0; j < lq; j++) row[j] = (u8)((pay[j] + h[j]) % q);
    }
}

/* Evaluate: the colour of the active label selects the row; subtract its hash. */
static void proj_eval_one(const octx *c, int p, int q, const u8 *in, int layer, uint32_t slot, u64 elem,
                          const u8 *rows, u8 *out) {
    int lq = c->lam[q], pitch = pitch_of(lq);
    u8 h[MAXLAM];
    hash(c, in, p, layer, slot, elem, q, h);
    const u8 *row = rows + (size_t)in[0] * pitch;
    for (int j = 0; j < lq; j++) out[j] = (u8)((row[j] + q - h[j]) % q);
}

/* A batch of n independent gates p -> q (the projection microbenchmark).  Gate g has
 * element index elem_base+g, its own table phi + g*phi_stride, a fresh output zero label
 * drawn from the PRG.  table: [g][p][pitch_q]. */
void orc_proj_garble(const octx *c, int p, int q, long n, u64 elem_base, int layer, uint32_t slot,
                     const u8 *in0, const u8 *phi, long phi_stride, u8 *out0, u8 *table) {
    int lp = c->lam[p], lq = c->lam[q];
    size_t tsz = (size_t)p * pitch_of(lq);
    for (long g = 0; g < n; g++) {
        draw(c, DOM_GATE, layer, slot, elem_base + (u64)g, q, out0 + g * lq);
        proj_garble_one(c, p, q, in0 + g * lp, phi + g * phi_stride, out0 + g * lq, layer, slot,
                        elem_base + (u64)g, table + g * tsz);
    }
}
void orc_proj_eval(const octx *c, int p, int q, long n, u64 elem_base, int layer, uint32_t slot,
                   const u8 *in, const u8 *table, u8 *out) {
    int lp = c->lam[p], lq = c->lam[q];
    size_t tsz = (size_t)p * pitch_of(lq);
    for (long g = 0; g < n; g++)
        proj_eval_one(c, p, q, in + g * lp, layer, slot, elem_base + (u64)g, table + g * tsz, out + g * lq);
}

/* ------------------------------------------------------------------------- */
/* Mixed-modulus half gate: z = a*b, a on a Z_p wire, b in {0,1} on a Z_2    */
/* wire (Appendix, Half-Gate Generalization and Mixed-Modulus Half-Gate).    */
/* ------------------------------------------------------------------------- */

/* Tables: G [p rows][pitch_p], E [2 rows][pitch_p], S [2 rows][4] (one digit each).
 * slots: slotG, slotG+1 (E), slotG+2 (S).  The mask r is drawn from the PRG
 * (domain MASK, slotG), the zero labels U0, V0 from domain GATE at slotG, slotG+1.
 *   G[colour(lx^a)] = U0 + a*r*R_p             + H_p(lx^a)
 *   E[colour(ly^b)] = V0 - (b+r)*lx^0          + H_p(ly^b)
 *   S[colour(ly^b)] = (b + r + H_p(ly^b)[0]) mod p
 * zero label of z: V0 - U0.  G == NULL: only z0 is produced (no ciphertexts). */
static void hg_garble_one(const octx *c, int p, const u8 *x0, const u8 *y0, int layer, uint32_t slotG,
                          u64 elem, u8 *z0, u8 *G, u8 *E, u8 *S) {
    int lp = c->lam[p], l2 = c->lam[2], pitch = pitch_of(lp);
    u8 U0[MAXLAM], V0[MAXLAM], rl[MAXLAM], la[MAXLAM], h[MAXLAM], pay[MAXLAM];
    draw(c, DOM_GATE, layer, slotG, elem, p, U0);
    draw(c, DOM_GATE, layer, slotG + 1, elem, p, V0);
    draw(c, DOM_MASK, layer, slotG, elem, p, rl);
    int r = rl[0];
    for (int a = 0; a < p && G; a++) {
        lab_axpy(la, x0, a, c->delta[p], lp, p);
        hash(c, la, p, layer, slotG, elem, p, h);
        lab_axpy(pay, U0, (long)a * r, c->delta[p], lp, p);
        u8 *row = G + (size_t)la[0] * pitch;
        memset(row, 0, (size_t)pitch);
        for (int j = 0; j < lp; j++) row[j] = (u8)((pay[j] + h[j]) % p);
    }
    for (int b = 0; b < 2 && G; b++) {
        lab_axpy(la, y0, b, c->delta[2], l2, 2);
        hash(c, la, 2, layer, slotG + 1, elem, p, h);
        lab_axpy(pay, V0, -(long)((b + r) % p), x0, lp, p);
        u8 *row = E + (size_t)la[0] * pitch;
        memset(row, 0, (size_t)pitch);
        for (int j = 0; j < lp; j++) row[j] = (u8)((pay[j] + h[j]) % p);
        hash(c, la, 2, layer, slotG + 2, elem, p, h);
        u8 *srow = S + (size_t)la[0] * 4;
        memset(srow, 0, 4);
        srow[0] = (u8)((b + r + h[0]) % p);
    }
    for (int j = 0; j < lp; j++) z0[j] = (u8)((V0[j] + p - U0[j]) % p);
}

/* Evaluator: U = G[..]-H, V = E[..]-H, beta = S[..]-H[0]; z = V + beta*lx - U. */
static void hg_eval_one(const octx *c, int p, const u8 *x, const u8 *y, int layer, uint32_t slotG, u64 elem,
                        const u8 *G, const u8 *E, const u8 *S, u8 *z) {
    int lp = c->lam[p], pitch = pitch_of(lp);
    u8 h[MAXLAM], U[MAXLAM], V[MAXLAM];
    hash(c, x, p, layer, slotG, elem, p, h);
    const u8 *row = G + (size_t)x[0] * pitch;
    for (int j = 0; j < lp; j++) U[j] = (u8)((row[j] + p - h[j]) % p);
    hash(c, y, 2, layer, slotG + 1, elem, p, h);
    row = E + (size_t)y[0] * pitch;
    for (int j = 0; j < lp; j++) V[j] = (u8)((row[j] + p - h[j]) % p);
    hash(c, y, 2, layer, slotG + 2, elem, p, h);
    int beta = (S[(size_t)y[0] * 4] + p - h[0]) % p;
    for (int j = 0; j < lp; j++) z[j] = (u8)((V[j] + (long)beta * x[j] + p - U[j]) % p);
}

void orc_hg_garble(const octx *c, int p, const u8 *x0, const u8 *y0, int layer, uint32_t slotG, u64 elem,
                   u8 *z0, u8 *G, u8 *E, u8 *S) { hg_garble_one(c, p, x0, y0, layer, slotG, elem, z0, G, E, S); }
void orc_hg_eval(const octx *c, int p, const u8 *x, const u8 *y, int layer, uint32_t slotG, u64 elem,
                 const u8 *G, const u8 *E, const u8 *S, u8 *z) { hg_eval_one(c, p, x, y, layer, slotG, elem, G, E, S, z); }

/* ------------------------------------------------------------------------- */
/* Approximated sign (Appendix, Approximated Garbled Sign + Garbled          */
/* Mixed-Radix Addition)                                                     */
/* ------------------------------------------------------------------------- */

/* phi_{i,j}(x): digit j (d_1 most significant) of ceil(M*u/p_i), u = x*(P/p_i)^{-1} mod p_i,
 * i.e. the fraction (alpha_i * x / P) mod 1 rounded UP to a multiple of 1/M.
 * With every term rounded up and M >= k*P the k-term sum overestimates the true
 * fraction X/P by less than 1/P, which never crosses 1/2 nor 1: the sign is exact. */
static int sign_phi(const octx *c, int i, int j, int x) {
    int p = c->prime[i];
    u64 A = c->P / (u64)p;
    int Am = (int)(A % (u64)p), inv = 0;
    for (int t = 1; t < p; t++) if ((Am * t) % p == 1) { inv = t; break; }
    int u = (x * inv) % p;
    u128 N = (c->M * (u128)u + (u128)(p - 1)) / (u128)p;       /* ceil(M*u/p) */
    u128 w = 1;
    for (int t = c->n; t > j; t--) w *= (u128)c->d[t];           /* weight of digit j */
    return (int)((N / w) % (u128)c->d[j]);
}
int orc_sign_phi(const octx *c, int i, int j, int x) { return sign_phi(c, i, j, x); }

/* Slot numbering inside one sign gadget with k residues and n digits:
 *   digit gate (i, j), i = 0..k-1, j = 1..n : i*n + (j-1)
 *   carry gate out of digit j, j = n..2     : k*n + (j-2)
 *   final gate                              : k*n + n-1
 * Every slot owns one table segment (rows = input modulus, width = output modulus);
 * a residue that is skipped (first_res = 1) owns no segment. */
static int sign_nslots(const octx *c) { return c->k * c->n + c->n; }
static int sign_slot_in(const octx *c, int s) {
    int k = c->k, n = c->n;
    if (s < k * n) return c->prime[s / n];
    if (s < k * n + n - 1) return c->mj[(s - k * n) + 2];
    return c->mj[1];
}
static int sign_slot_out(const octx *c, int s) {
    int k = c->k, n = c->n;
    if (s < k * n) return c->mj[(s % n) + 1];
    if (s < k * n + n - 1) return c->mj[(s - k * n) + 1];
    return 2;
}
/* bytes of table per element owned by sign slot s */
static size_t sign_slot_bytes(const octx *c, int s, int first_res) {
    if (s < c->k * c->n && s / c->n < first_res) return 0;
    return (size_t)sign_slot_in(c, s) * pitch_of(c->lam[sign_slot_out(c, s)]);
}

/* Garble / evaluate one sign gadget for ONE element.
 * x[i]      : zero (garble) or active (eval) label of residue i, i >= first_res
 * seg[s]    : this element's rows of slot s
 * negate=0  : output bit = [X >= P/2];  negate=1 : output bit = [X < P/2]
 * wires     : if not NULL, [sign_nslots][MAXLAM] receives the label of every gate output */
static void sign_garble_one(const octx *c, int first_res, int negate, u8 *const x0[], int layer,
                            uint32_t slot_base, u64 elem, u8 *const seg[], u8 *bit0, u8 *wires) {
    int k = c->k, n = c->n;
    u8 acc[MAXN + 1][MAXLAM];       /* running free sum of the digit wires of digit j */
    u8 phi[256], w0[MAXLAM];
    for (int j = 1; j <= n; j++) lab_zero(acc[j], MAXLAM);
    for (int i = first_res; i < k; i++)
        for (int j = 1; j <= n; j++) {
            int s = i * n + (j - 1), p = c->prime[i], m = c->mj[j];
            for (int a = 0; a < p; a++) phi[a] = (u8)sign_phi(c, i, j, a);
            draw(c, DOM_GATE, layer, slot_base + (uint32_t)s, elem, m, w0);
            proj_garble_one(c, p, m, x0[i], phi, w0, layer, slot_base + (uint32_t)s, elem, seg[s]);
            lab_axpy(acc[j], acc[j], 1, w0, c->lam[m], m);
            if (wires) memcpy(wires + (size_t)s * MAXLAM, w0, (size_t)c->lam[m]);
        }
    for (int j = n; j >= 2; j--) {  /* carry out of digit j into digit j-1 */
        int s = k * n + (j - 2), m = c->mj[j], mo = c->mj[j - 1];
        for (int a = 0; a < m; a++) phi[a] = (u8)((a / c->d[j]) % mo);
        draw(c, DOM_GATE, layer, slot_base + (uint32_t)s, elem, mo, w0);
        proj_garble_one(c, m, mo, acc[j], phi, w0, layer, slot_base + (uint32_t)s, elem, seg[s]);
        lab_axpy(acc[j - 1], acc[j - 1], 1, w0, c->lam[mo], mo);
        if (wires) memcpy(wires + (size_t)s * MAXLAM, w0, (size_t)c->lam[mo]);
    }
    {
        int s = k * n + n - 1, m = c->mj[1];
        for (int a = 0; a < m; a++) { int neg = (2 * a >= c->d[1]); phi[a] = (u8)(negate ? 1 - neg : neg); }
        draw(c, DOM_GATE, layer, slot_base + (uint32_t)s, elem, 2, bit0);
        proj_garble_one(c, m, 2, acc[1], phi, bit0, layer, slot_base + (uint32_t)s, elem, seg[s]);
        if (wires) memcpy(wires + (size_t)s * MAXLAM, bit0, (size_t)c->lam[2]);
    }
}

static void sign_eval_one(const octx *c, int first_res, u8 *const x[], int layer, uint32_t slot_base,
                          u64 elem, u8 *const seg[], u8 *bit, u8 *wires) {
    int k = c->k, n = c->n;
    u8 acc[MAXN + 1][MAXLAM], w[MAXLAM];
    for (int j = 1; j <= n; j++) lab_zero(acc[j], MAXLAM);
    for (int i = first_res; i < k; i++)
        for (int j = 1; j <= n; j++) {
            int s = i * n + (j - 1), p = c->prime[i], m = c->mj[j];
            proj_eval_one(c, p, m, x[i], layer, slot_base + (uint32_t)s, elem, seg[s], w);
            lab_axpy(acc[j], acc[j], 1, w, c->lam[m], m);
            if (wires) memcpy(wires + (size_t)s * MAXLAM, w, (size_t)c->lam[m]);
        }
    for (int j = n; j >= 2; j--) {
        int s = k * n + (j - 2), m = c->mj[j], mo = c->mj[j - 1];
        proj_eval_one(c, m, mo, acc[j], layer, slot_base + (uint32_t)s, elem, seg[s], w);
        lab_axpy(acc[j - 1], acc[j - 1], 1, w, c->lam[mo], mo);
        if (wires) memcpy(wires + (size_t)s * MAXLAM, w, (size_t)c->lam[mo]);
    }
    {
        int s = k * n + n - 1;
        proj_eval_one(c, c->mj[1], 2, acc[1], layer, slot_base + (uint32_t)s, elem, seg[s], bit);
        if (wires) memcpy(wires + (size_t)s * MAXLAM, bit, (size_t)c->lam[2]);
    }
}

/* The plain function the gadget computes, on residues: used by the brute-force pins. */
int orc_sign_plain(const octx *c, const int *res, int first_res, int negate) {
    int k = c->k, n = c->n, carry = 0, s1 = 0;
    for (int j = n; j >= 1; j--) {
        int s = carry;
        for (int i = first_res; i < k; i++) s += sign_phi(c, i, j, res[i]);
        s %= c->mj[j];
        if (j >= 2) carry = (s / c->d[j]) % c->mj[j - 1]; else s1 = s;
    }
    int neg = (2 * s1 >= c->d[1]);
    return negate ? 1 - neg : neg;
}

/* ------------------------------------------------------------------------- */
/* Table geometry of the activation layers                                   */
/* ------------------------------------------------------------------------- */

/* ReLU layer, per element: the sign slots, then per residue i the half-gate
 * segments G_i, E_i, S_i (slots nsign+3i, +1, +2). */
size_t orc_relu_bytes_per_elem(const octx *c) {
    size_t b = 0;
    for (int s = 0; s < sign_nslots(c); s++) b += sign_slot_bytes(c, s, 0);
    for (int i = 0; i < c->k; i++) {
        int p = c->prime[i], pitch = pitch_of(c->lam[p]);
        b += (size_t)p * pitch + 2 * (size_t)pitch + 8;
    }
    return b;
}
/* Scale-by-2 layer, per element and repetition: k-1 cast segments (2 rows, residue i
 * at local slot i-1), then the sign slots without residue 0 (local slot k-1+s). */
size_t orc_scale_bytes_per_elem(const octx *c) {
    size_t b = 0;
    for (int i = 1; i < c->k; i++) b += 2 * (size_t)pitch_of(c->lam[c->prime[i]]);
    for (int s = 0; s < sign_nslots(c); s++) b += sign_slot_bytes(c, s, 1);
    return b;
}
int orc_sign_nslots(const octx *c) { return sign_nslots(c); }

/* ------------------------------------------------------------------------- */
/* ReLU layer: a * sgn_{0,1}(a)  (Sec. Arithmetic Garbled Circuits, Sign      */
/* Gadget paragraph; System-level Architecture)                              */
/* ------------------------------------------------------------------------- */

/* in0[i], out0[i]: label tensors [n][lambda_{p_i}] of residue i.
 * tables: orc_relu_bytes_per_elem * n bytes, or NULL (garbler only): zero labels without
 * ciphertexts.  wires (optional): [n][nsign][MAXLAM]. */
void orc_relu_garble(const octx *c, int layer, u64 elem_base, long n, u8 *const in0[], u8 *const out0[],
                     u8 *tables, u8 *wires) {
    int k = c->k, ns = sign_nslots(c);
    size_t off[MAXK * MAXN + MAXN + 3 * MAXK + 1];
    size_t cum = 0;
    for (int s = 0; s < ns; s++) { off[s] = cum; cum += sign_slot_bytes(c, s, 0); }
    for (int i = 0; i < k; i++) {
        int pitch = pitch_of(c->lam[c->prime[i]]);
        off[ns + 3 * i] = cum;     cum += (size_t)c->prime[i] * pitch;
        off[ns + 3 * i + 1] = cum; cum += 2 * (size_t)pitch;
        off[ns + 3 * i + 2] = cum; cum += 8;
    }
    for (long e = 0; e < n; e++) {
        u8 *x0[MAXK], *seg[MAXK * MAXN + MAXN];
        u8 bit0[MAXLAM];
        for (int i = 0; i < k; i++) x0[i] = in0[i] + e * c->lam[c->prime[i]];
        for (int s = 0; s < ns; s++)
            seg[s] = tables ? tables + (size_t)n * off[s] + (size_t)e * sign_slot_bytes(c, s, 0) : NULL;
        /* pos = [X < P/2]; ReLU keeps X when pos = 1 */
        sign_garble_one(c, 0, 1, x0, layer, 0, elem_base + (u64)e, seg, bit0,
                        wires ? wires + (size_t)e * ns * MAXLAM : NULL);
        for (int i = 0; i < k; i++) {
            int p = c->prime[i], pitch = pitch_of(c->lam[p]);
            u8 *G = tables ? tables + (size_t)n * off[ns + 3 * i] + (size_t)e * p * pitch : NULL;
            u8 *E = tables ? tables + (size_t)n * off[ns + 3 * i + 1] + (size_t)e * 2 * pitch : NULL;
            u8 *S = tables ? tables + (size_t)n * off[ns + 3 * i + 2] + (size_t)e * 8 : NULL;
            hg_garble_one(c, p, x0[i], bit0, layer, (uint32_t)(ns + 3 * i), elem_base + (u64)e,
                          out0[i] + e * c->lam[p], G, E, S);
        }
    }
}

void orc_relu_eval(const octx *c, int layer, u64 elem_base, long n, u8 *const in[], const u8 *tables,
                   u8 *const out[], u8 *wires) {
    int k = c->k, ns = sign_nslots(c);
    size_t off[MAXK * MAXN + MAXN + 3 * MAXK + 1];
    size_t cum = 0;
    for (int s = 0; s < ns; s++) { off[s] = cum; cum += sign_slot_bytes(c, s, 0); }
    for (int i = 0; i < k; i++) {
        int pitch = pitch_of(c->lam[c->prime[i]]);
        off[ns + 3 * i] = cum;     cum += (size_t)c->prime[i] * pitch;
        off[ns + 3 * i + 1] = cum; cum += 2 * (size_t)pitch;
        off[ns + 3 * i + 2] = cum; cum += 8;
    }
    for (long e = 0; e < n; e++) {
        u8 *x[MAXK], *seg[MAXK * MAXN + MAXN];
        u8 bit[MAXLAM];
        for (int i = 0; i < k; i++) x[i] = in[i] + e * c->lam[c->prime[i]];
        for (int s = 0; s < ns; s++)
            seg[s] = (u8 *)tables + (size_t)n * off[s] + (size_t)e * sign_slot_bytes(c, s, 0);
        sign_eval_one(c, 0, x, layer, 0, elem_base + (u64)e, seg, bit,
                      wires ? wires + (size_t)e * ns * MAXLAM : NULL);
        for (int i = 0; i < k; i++) {
            int p = c->prime[i], pitch = pitch_of(c->lam[p]);
            const u8 *G = tables + (size_t)n * off[ns + 3 * i] + (size_t)e * p * pitch;
            const u8 *E = tables + (size_t)n * off[ns + 3 * i + 1] + (size_t)e * 2 * pitch;
            const u8 *S = tables + (size_t)n * off[ns + 3 * i + 2] + (size_t)e * 8;
            hg_eval_one(c, p, x[i], bit, layer, (uint32_t)(ns + 3 * i), elem_base + (u64)e, G, E, S,
                        out[i] + e * c->lam[p]);
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Scaling by 2, `repeat` times (Sec. The Scaling Operation)                 */
/* ------------------------------------------------------------------------- */

/* One repetition, garbler side (zero labels) or evaluator side (active labels), for ONE
 * element.  `one[i]` is the constant-one wire's zero label (garble) / active label (eval).
 *  (1) ShiftUp : add P/2, which is 1 mod 2 and 0 mod every odd prime.
 *  (2) Scale   : cast the mod-2 residue into Z_{p_i} (2-row gate), b_i = (x_i - cast_i) * 2^{-1}.
 *  (3) Base extension: the number with residues [0, b_1..b_{k-1}] is the halved value Y or
 *      Y + P/2; Y < P/2, so [.. >= P/2] is exactly the missing mod-2 residue of Y.
 *  (4) ShiftDown : subtract floor(P/4). */
static void scale_one(const octx *c, int garble, u8 *const xin[], u8 *const one[], int layer,
                      uint32_t slot_base, u64 elem, u8 *const castseg[], u8 *const signseg[],
                      u8 *const xout[]) {
    int k = c->k, l2 = c->lam[2];
    u8 up[MAXLAM], cast[MAXLAM], b[MAXK][MAXLAM], bit[MAXLAM];
    u8 *bp[MAXK];
    u8 phi_id[2] = {0, 1};
    lab_axpy(up, xin[0], 1, one[0], l2, 2);
    for (int i = 1; i < k; i++) {
        int p = c->prime[i], lp = c->lam[p];
        uint32_t slot = slot_base + (uint32_t)(i - 1);
        if (garble) {
            draw(c, DOM_GATE, layer, slot, elem, p, cast);
            proj_garble_one(c, 2, p, up, phi_id, cast, layer, slot, elem, castseg[i]);
        } else proj_eval_one(c, 2, p, up, layer, slot, elem, castseg[i], cast);
        int inv2 = (p + 1) / 2;
        u8 diff[MAXLAM];
        lab_axpy(diff, xin[i], -1, cast, lp, p);
        lab_zero(b[i], lp);
        lab_axpy(b[i], b[i], inv2, diff, lp, p);
        bp[i] = b[i];
    }
    bp[0] = NULL;
    if (garble) sign_garble_one(c, 1, 0, bp, layer, slot_base + (uint32_t)(k - 1), elem, signseg, bit, NULL);
    else sign_eval_one(c, 1, bp, layer, slot_base + (uint32_t)(k - 1), elem, signseg, bit, NULL);
    u64 quarter = c->P / 4;
    lab_axpy(xout[0], bit, -(long)(quarter % 2), one[0], l2, 2);
    for (int i = 1; i < k; i++) {
        int p = c->prime[i];
        lab_axpy(xout[i], b[i], -(long)(quarter % (u64)p), one[i], c->lam[p], p);
    }
}

static void scale_layer(const octx *c, int garble, int layer, u64 elem_base, long n, int repeat,
                        u8 *const in[], u8 *tables, u8 *const out[]) {
    int k = c->k, ns = sign_nslots(c);
    size_t bpe = orc_scale_bytes_per_elem(c);
    size_t coff[MAXK], soff[MAXK * MAXN + MAXN], cum = 0;
    for (int i = 1; i < k; i++) { coff[i] = cum; cum += 2 * (size_t)pitch_of(c->lam[c->prime[i]]); }
    for (int s = 0; s < ns; s++) { soff[s] = cum; cum += sign_slot_bytes(c, s, 1); }
    uint32_t slots_per_rep = (uint32_t)(k - 1 + ns);
    u8 onebuf[MAXK][MAXLAM];
    u8 *one[MAXK];
    for (int i = 0; i < k; i++) {
        int p = c->prime[i];
        if (garble) memcpy(onebuf[i], c->one0[i], (size_t)c->lam[p]);
        else lab_axpy(onebuf[i], c->one0[i], 1, c->delta[p], c->lam[p], p);
        one[i] = onebuf[i];
    }
    for (long e = 0; e < n; e++) {
        u8 cur[MAXK][MAXLAM], nxt[MAXK][MAXLAM];
        u8 *curp[MAXK], *nxtp[MAXK];
        for (int i = 0; i < k; i++) {
            memcpy(cur[i], in[i] + e * c->lam[c->prime[i]], (size_t)c->lam[c->prime[i]]);
            curp[i] = cur[i]; nxtp[i] = nxt[i];
        }
        for (int t = 0; t < repeat; t++) {
            u8 *castseg[MAXK], *signseg[MAXK * MAXN + MAXN];
            u8 *rep = tables ? tables + (size_t)t * (size_t)n * bpe : NULL;     /* NULL (garbler): no ciphertexts */
            for (int i = 1; i < k; i++)
                castseg[i] = rep ? rep + (size_t)n * coff[i] + (size_t)e * 2 * pitch_of(c->lam[c->prime[i]]) : NULL;
            for (int s = 0; s < ns; s++)
                signseg[s] = rep ? rep + (size_t)n * soff[s] + (size_t)e * sign_slot_bytes(c, s, 1) : NULL;
            scale_one(c, garble, curp, one, layer, (uint32_t)t * slots_per_rep, elem_base + (u64)e,
                      castseg, signseg, nxtp);
            for (int i = 0; i < k; i++) memcpy(cur[i], nxt[i], (size_t)c->lam[c->prime[i]]);
        }
        for (int i = 0; i < k; i++) memcpy(out[i] + e * c->lam[c->prime[i]], cur[i], (size_t)c->lam[c->prime[i]]);
    }
}

void orc_scale_garble(const octx *c, int layer, u64 elem_base, long n, int repeat, u8 *const in0[],
                      u8 *tables, u8 *const out0[]) { scale_layer(c, 1, layer, elem_base, n, repeat, in0, tables, out0); }
void orc_scale_eval(const octx *c, int layer, u64 elem_base, long n, int repeat, u8 *const in[],
                    const u8 *tables, u8 *const out[]) { scale_layer(c, 0, layer, elem_base, n, repeat, in, (u8 *)tables, out); }

/* ------------------------------------------------------------------------- */
/* Sign activation sgn_{-1,1} (Sec. Arithmetic Garbled Circuits, Sign Gadget) */
/* ------------------------------------------------------------------------- */

/* The gadget's bit neg = [X >= P/2] is cast into every residue by a 2-row gate
 * (local slot nsign + i) with phi(0) = 1, phi(1) = -1 mod p_i: output +1 for X in the
 * lower half (zero included), -1 for the upper half. */
size_t orc_signact_bytes_per_elem(const octx *c) {
    size_t b = 0;
    for (int s = 0; s < sign_nslots(c); s++) b += sign_slot_bytes(c, s, 0);
    for (int i = 0; i < c->k; i++) b += 2 * (size_t)pitch_of(c->lam[c->prime[i]]);
    return b;
}
static void signact_layer(const octx *c, int garble, int layer, u64 elem_base, long n, u8 *const in[],
                          u8 *tables, u8 *const out[]) {
    int k = c->k, ns = sign_nslots(c);
    size_t off[MAXK * MAXN + MAXN + MAXK], cum = 0;
    for (int s = 0; s < ns; s++) { off[s] = cum; cum += sign_slot_bytes(c, s, 0); }
    for (int i = 0; i < k; i++) { off[ns + i] = cum; cum += 2 * (size_t)pitch_of(c->lam[c->prime[i]]); }
    for (long e = 0; e < n; e++) {
        u8 *x[MAXK], *seg[MAXK * MAXN + MAXN];
        u8 bit[MAXLAM];
        for (int i = 0; i < k; i++) x[i] = in[i] + e * c->lam[c->prime[i]];
        for (int s = 0; s < ns; s++) seg[s] = tables + (size_t)n * off[s] + (size_t)e * sign_slot_bytes(c, s, 0);
        if (garble) sign_garble_one(c, 0, 0, x, layer, 0, elem_base + (u64)e, seg, bit, NULL);
        else sign_eval_one(c, 0, x, layer, 0, elem_base + (u64)e, seg, bit, NULL);
        for (int i = 0; i < k; i++) {
            int p = c->prime[i], lp = c->lam[p];
            u8 phi[2] = {1, (u8)(p - 1)};
            if (p == 2) phi[1] = 1;
            u8 *rows = tables + (size_t)n * off[ns + i] + (size_t)e * 2 * pitch_of(lp);
            u8 *o = out[i] + e * lp;
            if (garble) {
                draw(c, DOM_GATE, layer, (uint32_t)(ns + i), elem_base + (u64)e, p, o);
                proj_garble_one(c, 2, p, bit, phi, o, layer, (uint32_t)(ns + i), elem_base + (u64)e, rows);
            } else proj_eval_one(c, 2, p, bit, layer, (uint32_t)(ns + i), elem_base + (u64)e, rows, o);
        }
    }
}
void orc_signact_garble(const octx *c, int layer, u64 elem_base, long n, u8 *const in0[], u8 *tables,
                        u8 *const out0[]) { signact_layer(c, 1, layer, elem_base, n, in0, tables, out0); }
void orc_signact_eval(const octx *c, int layer, u64 elem_base, long n, u8 *const in[], const u8 *tables,
                      u8 *const out[]) { signact_layer(c, 0, layer, elem_base, n, in, (u8 *)tables, out); }

/* ------------------------------------------------------------------------- */
/* Packed storage format of the ciphertext tables                            */
/* ------------------------------------------------------------------------- */

/* A ciphertext is an encrypted label, a vector in Z_q^lambda_q; for storage and transfer it is
 * compressed like a label (Sec. Implementation, compress; Sec. Evaluation, Communication: labels
 * travel as 128 bits): 16 bytes per row, little endian, in place of pitch_q.  The one-digit rows of
 * a half gate (4 bytes in the working format) take one byte.  Segments keep their order; a
 * one-digit segment is padded to a multiple of 16 bytes.  Only defined when q^lambda_q <= 2^128 for
 * every row modulus of the layer (the floor rule); returns 0 otherwise.
 * kind: 4 ReLU, 5 scaling (repeat), 6 sign activation, 7 one segment of gates p -> q. */
typedef struct { int rows, q; } oseg;      /* rows per element, modulus of the rows (0: one-digit rows) */
static int table_segments(const octx *c, int kind, int repeat, int p, int q, oseg *out) {
    int n = 0, k = c->k, ns = sign_nslots(c);
    int reps = kind == 5 ? repeat : 1;
    for (int t = 0; t < reps; t++) {
        if (kind == 5) for (int i = 1; i < k; i++) out[n++] = (oseg){2, c->prime[i]};
        if (kind == 4 || kind == 5 || kind == 6)
            for (int s = 0; s < ns; s++)
                if (sign_slot_bytes(c, s, kind == 5)) out[n++] = (oseg){sign_slot_in(c, s), sign_slot_out(c, s)};
        if (kind == 4) for (int i = 0; i < k; i++) {
            out[n++] = (oseg){c->prime[i], c->prime[i]};
            out[n++] = (oseg){2, c->prime[i]};
            out[n++] = (oseg){2, 0};
        }
        if (kind == 6) for (int i = 0; i < k; i++) out[n++] = (oseg){2, c->prime[i]};
        if (kind == 7) out[n++] = (oseg){p, q};
    }
    return n;
}
static int row_fits_128(const octx *c, int q) {
    u128 v = 1;
    for (int j = 0; j < c->lam[q]; j++) {
        if (v > (~(u128)0) / (u128)q) return (q == 2 || q == 4 || q == 16) && j == c->lam[q] - 1;   /* q^lambda = 2^128 exactly */
        v *= (u128)q;
    }
    return 1;
}
#define MAXSEG (MAXN * (MAXK * MAXN + MAXN + MAXK) + 4 * MAXK + 8)
size_t orc_tables_packed_bytes(const octx *c, int kind, long n, int repeat, int p, int q) {
    oseg seg[MAXSEG];
    int ns = table_segments(c, kind, repeat, p, q, seg);
    size_t b = 0;
    for (int s = 0; s < ns; s++) {
        if (seg[s].q && !row_fits_128(c, seg[s].q)) return 0;
        b += seg[s].q ? (size_t)n * seg[s].rows * 16 : (((size_t)n * seg[s].rows + 15) / 16) * 16;
    }
    return b;
}
/* pack = 1: tables -> packed; pack = 0: packed -> tables.  Returns 0 if the format is not defined. */
int orc_tables_repack(const octx *c, int kind, long n, int repeat, int p, int q, int pack, u8 *tables, u8 *packed) {
    oseg seg[MAXSEG];
    int ns = table_segments(c, kind, repeat, p, q, seg);
    if (!orc_tables_packed_bytes(c, kind, n, repeat, p, q) && ns && n) return 0;
    for (int s = 0; s < ns; s++) {
        size_t rows = (size_t)n * seg[s].rows;
        if (!seg[s].q) {
            for (size_t r = 0; r < rows; r++) {
                if (pack) packed[r] = tables[4 * r];
                else { memset(tables + 4 * r, 0, 4); tables[4 * r] = packed[r]; }
            }
            if (pack) memset(packed + rows, 0, ((rows + 15) / 16) * 16 - rows);
            tables += 4 * rows; packed += ((rows + 15) / 16) * 16;
            continue;
        }
        int lq = c->lam[seg[s].q], pitch = pitch_of(lq);
        for (size_t r = 0; r < rows; r++) {
            u8 *row = tables + r * pitch, *pk = packed + r * 16;
            if (pack) store128(compress(row, lq, seg[s].q), pk);
            else { memset(row, 0, (size_t)pitch); decompress(load128(pk), seg[s].q, lq, row); }
        }
        tables += rows * pitch; packed += rows * 16;
    }
    return 1;
}

/* ------------------------------------------------------------------------- */
/* Linear layers: free additions and multiplications by public constants     */
/* (Sec. Arithmetic Garbled Circuits; System-level Architecture; LabelTensors */
/* figure of the Conv2D operation)                                           */
/* ------------------------------------------------------------------------- */

/* Tensors of one batch element are stored [y][x][channel]; conv weights
 * [out_c][ky][kx][in_c]; a dense layer is a 1x1 "image" with in_c = K inputs.
 * out[b][oy][ox][co] = sum W[co][ky][kx][ci] * in[b][oy*stride+ky-pad][ox*stride+kx-pad][ci]
 *                      (+ bias[co] * one), per label component, mod p.
 * Positions outside the image contribute nothing.  The same routine serves the garbler
 * (zero labels, one = zero label of the constant wire) and the evaluator. */
void orc_conv2d(const octx *c, int i, long batch, int in_h, int in_w, int in_c, int out_c, int kh, int kw,
                int stride, int pad, const int32_t *W, const int32_t *bias, const u8 *one,
                const u8 *in, u8 *out) {
    int p = c->prime[i], lam = c->lam[p];
    int out_h = (in_h + 2 * pad - kh) / stride + 1, out_w = (in_w + 2 * pad - kw) / stride + 1;
    for (long b = 0; b < batch; b++)
        for (int oy = 0; oy < out_h; oy++)
            for (int ox = 0; ox < out_w; ox++)
                for (int co = 0; co < out_c; co++) {
                    u64 acc[MAXLAM];
                    for (int d = 0; d < lam; d++) acc[d] = 0;
                    for (int ky = 0; ky < kh; ky++)
                        for (int kx = 0; kx < kw; kx++) {
                            int iy = oy * stride + ky - pad, ix = ox * stride + kx - pad;
                            if (iy < 0 || iy >= in_h || ix < 0 || ix >= in_w) continue;
                            for (int ci = 0; ci < in_c; ci++) {
                                long w = W[(((size_t)co * kh + ky) * kw + kx) * in_c + ci];
                                u64 wm = (u64)(((w % p) + p) % p);
                                const u8 *l = in + ((((size_t)b * in_h + iy) * in_w + ix) * in_c + ci) * lam;
                                for (int d = 0; d < lam; d++) acc[d] += wm * l[d];
                            }
                        }
                    u8 *o = out + ((((size_t)b * out_h + oy) * out_w + ox) * out_c + co) * lam;
                    u64 bm = bias ? (u64)(((bias[co] % p) + p) % p) : 0;
                    for (int d = 0; d < lam; d++) o[d] = (u8)((acc[d] + (bias ? bm * one[d] : 0)) % (u64)p);
                }
}

/* 2x2 sum-pool, stride 2 (a convolution with weights 1): free additions. */
void orc_sumpool2(const octx *c, int i, long batch, int in_h, int in_w, int ch, const u8 *in, u8 *out) {
    int p = c->prime[i], lam = c->lam[p], oh = in_h / 2, ow = in_w / 2;
    for (long b = 0; b < batch; b++)
        for (int oy = 0; oy < oh; oy++)
            for (int ox = 0; ox < ow; ox++)
                for (int ch_i = 0; ch_i < ch; ch_i++) {
                    u8 *o = out + ((((size_t)b * oh + oy) * ow + ox) * ch + ch_i) * lam;
                    for (int d = 0; d < lam; d++) {
                        int s = 0;
                        for (int dy = 0; dy < 2; dy++)
                            for (int dx = 0; dx < 2; dx++)
                                s += in[((((size_t)b * in_h + 2 * oy + dy) * in_w + 2 * ox + dx) * ch + ch_i) * lam + d];
                        o[d] = (u8)(s % p);
                    }
                }
}

/* ------------------------------------------------------------------------- */
/* En / De (Sec. Garbled Circuits: Gb, En, Ev, De; Sec. Quantization and      */
/* Encoding: Encode(x) = x mod P, negatives in the upper half)               */
/* ------------------------------------------------------------------------- */

void orc_encode(const octx *c, int i, long n, const int64_t *values, const u8 *zero, u8 *out) {
    int p = c->prime[i], lam = c->lam[p];
    for (long e = 0; e < n; e++) {
        long v = (long)(((values[e] % p) + p) % p);
        lab_axpy(out + e * lam, zero + e * lam, v, c->delta[p], lam, p);
    }
}

/* act[i], zero[i]: [n][lambda_{p_i}].  A label that is not zero + a*R for the a its colour
 * names is a forgery: valid[e] = 0 and values[e] = 0. */
void orc_decode(const octx *c, long n, u8 *const act[], u8 *const zero[], int64_t *values, u8 *valid) {
    int k = c->k;
    for (long e = 0; e < n; e++) {
        int ok = 1;
        int res[MAXK];
        for (int i = 0; i < k; i++) {
            int p = c->prime[i], lam = c->lam[p];
            const u8 *a = act[i] + e * lam, *z = zero[i] + e * lam;
            int v = (a[0] + p - z[0]) % p;       /* colour difference; R's colour is 1 */
            for (int j = 0; j < lam; j++)
                if (a[j] != (z[j] + v * c->delta[p][j]) % p) ok = 0;
            res[i] = v;
        }
        int64_t X = 0;
        if (ok) {
            /* CRT by search-free reconstruction: X = sum res_i * A_i * (A_i^{-1} mod p_i) mod P */
            u128 acc = 0;
            for (int i = 0; i < k; i++) {
                int p = c->prime[i];
                u64 A = c->P / (u64)p;
                int Am = (int)(A % (u64)p), inv = 0;
                for (int t = 1; t < p; t++) if ((Am * t) % p == 1) { inv = t; break; }
                acc += (u128)A * (u128)((res[i] * inv) % p);
            }
            u64 Xu = (u64)(acc % (u128)c->P);
            X = (2 * Xu >= c->P) ? (int64_t)Xu - (int64_t)c->P : (int64_t)Xu;
        }
        values[e] = X;
        valid[e] = (u8)ok;
    }
}
