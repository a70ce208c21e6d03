"""Analytic count of arithmetic operations and of bytes moved for the ABED schemes and their
implementation options (the estimation of Sec. 5.1, whose results are Sec. 6.1): implementation
details are abstracted away; a multiplication, an addition, a fused multiply-add, an activation
and a type cast each count as one operation; bytes are the inputs and outputs of every kernel an
option launches (Sec. 4.3).  No GPU is involved.

  python -m paper_2006_04984_amd.model --config 2        one JSON object: per layer and in total

Counts follow the schemes as this library implements them (d_f / d_i checksum digits, Sec. 4.1);
`granule` = the same with the checksum filters costed as a whole block of 16 filters, which is what
they occupy on the matrix units here (the paper adds 8 filters for the same reason, Sec. 5.2)."""
import argparse
import json


def digits_for_count(count):
    d, reach = 1, 1
    while count > reach:
        reach = reach * 256 + 1
        d += 1
    return d


def ops(s, int8_out=True):
    """Operation counts of one layer per scheme: dict scheme -> dict(part -> ops)."""
    npq, crs = s.N * s.P * s.Q, s.C * s.R * s.S
    outs = npq * s.K
    d_f, d_i = digits_for_count(s.K), digits_for_count(s.N)
    epilog = 5 * outs if int8_out else 0          # cast, scale, bias, activation, clamp + cast
    base = dict(convolution=outs * crs, epilog=epilog)
    fc = dict(convolution=npq * (s.K + d_f) * crs, epilog=epilog,
              output_checksum=npq * (s.K - 1) + npq * d_f,        # sum over k, recombine the digit fmaps
              verification=npq)
    fc_granule = dict(fc, convolution=npq * (s.K + 16) * crs)
    ic = dict(convolution=(s.N + d_i) * s.P * s.Q * s.K * crs, epilog=epilog,
              input_checksum=(s.N - 1) * s.H * s.W * s.C,
              output_checksum=(s.N - 1) * s.P * s.Q * s.K + s.P * s.Q * s.K * d_i,
              verification=s.P * s.Q * s.K)
    fic = dict(convolution=outs * crs, epilog=epilog,
               input_checksum=npq * crs,                            # PQNCRS additions (Sec. 3.3)
               dot_product=crs,
               output_checksum=outs,
               verification=1)
    ic2 = dict(convolution=outs * crs, epilog=epilog, input_checksum=npq * crs,
               checksum_convolution=crs * s.K, output_checksum=outs, verification=s.K)
    return dict(baseline=base, fc=fc, fc_granule=fc_granule, ic_batch=ic, fic=fic, ic2=ic2)


def moved_bytes(s, int8_out=True):
    """Bytes that form the inputs and outputs of all kernels of an option: dict option -> bytes."""
    npq, crs = s.N * s.P * s.Q, s.C * s.R * s.S
    x, w, outs = s.N * s.H * s.W * s.C, s.K * crs, npq * s.K
    d_f = digits_for_count(s.K)
    out_b = outs * (1 if int8_out else 4)
    fused = x + w + out_b                                            # convolution + epilog in one kernel
    unfused = x + w + 4 * outs + (4 * outs + out_b if int8_out else 0)   # ConvOut written, read by the epilog
    return dict(
        baseline_fused=fused,
        baseline_unfused=unfused,
        # FC: d_f extra filters and fmaps; unfused = a checksum kernel re-reads ConvOut, a compare kernel its results
        fc_unfused=unfused + d_f * crs + 4 * npq * d_f + (4 * outs + 4 * npq) + (4 * npq + 4 * npq * d_f),
        fc_fused=fused + d_f * crs + 4,                              # checksums made and compared in the kernel; a flag
        # FIC: input checksum kernel reads x once more; unfused = output checksum kernel re-reads ConvOut
        fic_unfused=unfused + (x + 4 * crs) + 4 * crs + 4 * outs + 8 + 2 * 4 * crs + 8,
        fic_fused=fused + (x + 4 * crs) + 4 * crs + 8 + 8,
    )


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2, choices=[2, 3, 5])
    ap.add_argument("--batch", type=int, default=0)
    args = ap.parse_args()
    from synth import CONFIG2, CONFIG3, resnet50_layers
    layers = {2: CONFIG2, 3: CONFIG3, 5: resnet50_layers(args.batch or 128)}[args.config]
    if args.batch and args.config != 5:
        import dataclasses
        layers = [dataclasses.replace(s, N=args.batch) for s in layers]
    tot_ops, tot_bytes, rows = {}, {}, []
    for s in layers:
        o, b = ops(s), moved_bytes(s)
        base = sum(o["baseline"].values())
        rows.append(dict(layer=s.name,
                         ops_increase_pct={k: 100.0 * (sum(v.values()) / base - 1.0) for k, v in o.items() if k != "baseline"},
                         bytes_vs_fused_baseline={k: v / b["baseline_fused"] for k, v in b.items()}))
        for k, v in o.items():
            tot_ops[k] = tot_ops.get(k, 0) + sum(v.values())
        for k, v in b.items():
            tot_bytes[k] = tot_bytes.get(k, 0) + v
    print(json.dumps(dict(config=args.config, batch=layers[0].N,
                          total_ops_increase_pct={k: 100.0 * (v / tot_ops["baseline"] - 1.0) for k, v in tot_ops.items() if k != "baseline"},
                          total_bytes_vs_fused_baseline={k: v / tot_bytes["baseline_fused"] for k, v in tot_bytes.items()},
                          layers=rows)))


if __name__ == "__main__":
    main()
