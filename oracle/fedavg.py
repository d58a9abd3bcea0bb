"""Mask handling, plaintext FedAvg and the end-to-end round (oracle side).

The selective-encryption mask M splits each flattened model into the part
that is encrypted, M . W, and the plaintext remainder (1-M) . W
(Algorithm 1; Section "Algorithm for HE-Based Federated Aggregation").
A mask is given as sorted disjoint runs (start, length).  The masked
parameters are packed in parameter order, n per ciphertext, the last
ciphertext zero-padded (a vector shorter than the packing batch still takes
a full ciphertext, Section "Results on Different Scales of Models"); the
remainder is kept compacted, in parameter order.

Plain FedAvg is W_glob = sum_i alpha_i W_i (Section "Federated Learning"),
evaluated in float64 in client order, acc <- acc + alpha_i * w (product and
sum rounded separately), with a single final rounding to float32.
"""
from __future__ import annotations

import numpy as np

from . import encoder, scheme
from .params import Params


def mask_indices(P: int, runs):
    """(enc_idx, plain_idx): parameter indices of the masked part and of the rest."""
    m = np.zeros(P, dtype=bool)
    prev_end = 0
    for start, length in runs:
        assert length > 0 and start >= prev_end and start + length <= P
        m[start:start + length] = True
        prev_end = start + length
    idx = np.arange(P, dtype=np.int64)
    return idx[m], idx[~m]


def n_ciphertexts(p: Params, n_enc: int) -> int:
    return -(-n_enc // p.n_slots)


def pack_slots(p: Params, w, enc_idx, ct_index: int):
    """Slot vector (float64, length n) of ciphertext `ct_index`, zero padded."""
    n = p.n_slots
    sel = enc_idx[ct_index * n:(ct_index + 1) * n]
    z = np.zeros(n, dtype=np.float64)
    z[:sel.shape[0]] = np.asarray(w)[sel].astype(np.float64)
    return z


def plain_fedavg(ws, alpha):
    """float32 result of the float64 weighted sum in client order."""
    acc = np.zeros(np.asarray(ws[0]).shape, dtype=np.float64)
    for a, w in zip(alpha, ws):
        acc = acc + np.float64(a) * np.asarray(w).astype(np.float64)
    return acc.astype(np.float32)


def fedavg_float64(ws, alpha):
    """The plain definition the whole method approximates: sum_i alpha_i W_i in float64."""
    acc = np.zeros(np.asarray(ws[0]).shape, dtype=np.float64)
    for a, w in zip(alpha, ws):
        acc = acc + np.float64(a) * np.asarray(w).astype(np.float64)
    return acc


def encrypt_ct(p, keys, w, enc_idx, seed, client_id, ct_index, fast=True):
    """Client side for one ciphertext: pack, encode, encrypt. Returns (m, ct)."""
    z = pack_slots(p, w, enc_idx, ct_index)
    enc = encoder.encode_fft if fast else encoder.encode_def
    m = enc(z, p.log2_n, p.scale_bits)
    return m, scheme.encrypt(p, keys, m, seed, client_id, ct_index)


def decode_ct(p, keys, ct_glob, fast=True):
    """Client side for one aggregated ciphertext: decrypt, lift, decode -> n float64 slots."""
    v = scheme.decrypt(p, keys, ct_glob, p.n_limbs - 1)
    dec = encoder.decode_fft if fast else encoder.decode_def
    return dec(np.array([float(x) for x in v], dtype=np.float64), p.log2_n, p.scale_bits)


def secure_round(p: Params, keys, ws, alpha, runs, seed, fast=True):
    """Whole round for K clients on the CPU.  Returns the merged float32 global model."""
    P = np.asarray(ws[0]).shape[0]
    enc_idx, plain_idx = mask_indices(P, runs)
    n_ct = n_ciphertexts(p, enc_idx.shape[0])
    out = np.zeros(P, dtype=np.float32)
    out[plain_idx] = plain_fedavg([np.asarray(w)[plain_idx] for w in ws], alpha)
    for c in range(n_ct):
        cts = [encrypt_ct(p, keys, w, enc_idx, seed, i, c, fast)[1] for i, w in enumerate(ws)]
        z = decode_ct(p, keys, scheme.aggregate(p, cts, alpha), fast)
        sel = enc_idx[c * p.n_slots:(c + 1) * p.n_slots]
        out[sel] = z[:sel.shape[0]].astype(np.float32)
    return out


# ---- variant: weighing on the client, the server only adds -------------------------------------
# (Section "Comparison with Other FL Frameworks" describes a system in which every learner multiplies
#  its own parameters by its weight before encrypting; no ciphertext-scalar product, no rescale.)

def encrypt_ct_weighted(p, keys, w, enc_idx, alpha_i, seed, client_id, ct_index, fast=True):
    """Client side: slots alpha_i * w (float64 product), encode, encrypt.  Returns (m, ct)."""
    z = np.float64(alpha_i) * pack_slots(p, w, enc_idx, ct_index)
    enc = encoder.encode_fft if fast else encoder.encode_def
    m = enc(z, p.log2_n, p.scale_bits)
    return m, scheme.encrypt(p, keys, m, seed, client_id, ct_index)


def plain_weighted(w, alpha_i):
    """What a client sends of its plaintext remainder: float32(alpha_i * w), product in float64."""
    return (np.float64(alpha_i) * np.asarray(w).astype(np.float64)).astype(np.float32)


def plain_sum(ws):
    """Server side of the plaintext remainder: float64 sum in client order, one rounding to float32."""
    acc = np.zeros(np.asarray(ws[0]).shape, dtype=np.float64)
    for w in ws:
        acc = acc + np.asarray(w).astype(np.float64)
    return acc.astype(np.float32)


def decode_ct_level(p, keys, ct_glob, level, fast=True):
    v = scheme.decrypt(p, keys, ct_glob, level)
    dec = encoder.decode_fft if fast else encoder.decode_def
    return dec(np.array([float(x) for x in v], dtype=np.float64), p.log2_n, p.scale_bits)


def secure_round_client_weighted(p: Params, keys, ws, alpha, runs, seed, fast=True):
    """Whole round of the variant for K clients.  Returns the merged float32 global model."""
    P = np.asarray(ws[0]).shape[0]
    enc_idx, plain_idx = mask_indices(P, runs)
    n_ct = n_ciphertexts(p, enc_idx.shape[0])
    out = np.zeros(P, dtype=np.float32)
    out[plain_idx] = plain_sum([plain_weighted(np.asarray(w)[plain_idx], a) for w, a in zip(ws, alpha)])
    for c in range(n_ct):
        cts = [encrypt_ct_weighted(p, keys, w, enc_idx, a, seed, i, c, fast)[1] for i, (w, a) in enumerate(zip(ws, alpha))]
        z = decode_ct_level(p, keys, scheme.sum_ciphertexts(p, cts), p.n_limbs, fast)
        sel = enc_idx[c * p.n_slots:(c + 1) * p.n_slots]
        out[sel] = z[:sel.shape[0]].astype(np.float32)
    return out


def noise_sigma_client_weighted(p: Params, n_clients: int):
    """Predicted RMS slot error of the variant: K fresh noises add up unweighted, no rescale term;
    each client's encoding rounding (variance 1/12 per coefficient) adds up as well."""
    half_eta = p.cbd_eta / 2.0
    var_fresh = half_eta * (2.0 / 3.0) * p.N * 2.0 + half_eta
    var_coeff = n_clients * (var_fresh + 1.0 / 12.0)
    return float(np.sqrt(p.N * var_coeff / 2.0)) / p.delta


def noise_sigma(p: Params, alpha):
    """Predicted RMS slot error of the decoded aggregate against exact FedAvg.

    Fresh-encryption noise e*u + e0 + e1*s has coefficient variance about
    (eta/2)*(2/3)*N*2 + eta/2; a slot sums N coefficients against cosines
    (mean square 1/2).  Averaging scales it by sum(alpha^2).  Rescale rounding
    tau0 + tau1*s adds variance (1 + 2N/3)/12 per coefficient.
    """
    n_ring = p.N
    half_eta = p.cbd_eta / 2.0
    var_fresh = half_eta * (2.0 / 3.0) * n_ring * 2.0 + half_eta
    var_coeff = var_fresh * float(np.sum(np.asarray(alpha, dtype=np.float64) ** 2)) \
        + (1.0 + 2.0 * n_ring / 3.0) / 12.0 + 1.0 / 12.0
    return float(np.sqrt(n_ring * var_coeff / 2.0)) / p.delta


def packed_to_param(starts, lens, t):
    """Parameter index of packed positions t (array) under the run list (starts, lens).

    Same map as mask_indices()[0][t], computed from the runs' prefix sums, so that it also
    works for vectors too long to enumerate."""
    starts = np.asarray(starts, dtype=np.int64)
    lens = np.asarray(lens, dtype=np.int64)
    prefix = np.concatenate([[0], np.cumsum(lens)])
    t = np.asarray(t, dtype=np.int64)
    assert t.size == 0 or (t.min() >= 0 and t.max() < prefix[-1])
    r = np.searchsorted(prefix, t, side="right") - 1
    return starts[r] + (t - prefix[r])


def complement_runs(P: int, starts, lens):
    """Run list of the unmasked remainder."""
    out_s, out_l, pos = [], [], 0
    for s, ln in zip(starts, lens):
        s, ln = int(s), int(ln)
        if s > pos:
            out_s.append(pos)
            out_l.append(s - pos)
        pos = s + ln
    if pos < P:
        out_s.append(pos)
        out_l.append(P - pos)
    return np.asarray(out_s, dtype=np.int64), np.asarray(out_l, dtype=np.int64)
