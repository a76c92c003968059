"""What the vendor's GEMM (torch.matmul -> hipBLASLt) reaches on this GPU at the shapes of the lowered CaffeNet
layers, with the lowered matrix already in memory: a yardstick for the library's own kernels, not part of any
product path (nothing in the library calls a vendor GEMM).  bf16, fp32 accumulation, random N(0,1) and all-zero
operands (the matrix cores draw less power on zeros and the chip clocks higher).

    python -m paper_1606_04487_amd.gemm_yardstick
"""
import torch
def bench(fn, n=20):
    for _ in range(3): fn()
    torch.cuda.synchronize()
    s=torch.cuda.Event(enable_timing=True); e=torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(n): fn()
    e.record(); torch.cuda.synchronize()
    return s.elapsed_time(e)/n
shapes = {"sq8192": (8192,8192,8192), "sq4096": (4096,4096,4096),
  "conv2_fwd": (256,186624,2400), "conv3_fwd": (384,43264,2304), "conv4_fwd": (384,43264,3456), "conv5_fwd": (256,43264,3456),
  "conv2_wgrad": (256,2400,186624), "conv4_wgrad": (384,3456,43264), "conv1_fwd": (96, 774400, 363)}
for dist in ("randn", "zeros"):
  for name,(m,n,k) in shapes.items():
    if dist=="randn":
        a=torch.randn(m,k,device="cuda",dtype=torch.bfloat16); b=torch.randn(k,n,device="cuda",dtype=torch.bfloat16)
    else:
        a=torch.zeros(m,k,device="cuda",dtype=torch.bfloat16); b=torch.zeros(k,n,device="cuda",dtype=torch.bfloat16)
    c=torch.empty(m,n,device="cuda",dtype=torch.bfloat16)
    ms=bench(lambda: torch.matmul(a,b,out=c))
    bt=b.t().contiguous()
    ms2=bench(lambda: torch.matmul(a,bt.t(),out=c))
    print(f"{dist} {name} {m}x{n}x{k}: NN {ms*1e3:.1f} us {2*m*n*k/ms/1e9:.0f} TF/s | NT {ms2*1e3:.1f} us {2*m*n*k/ms2/1e9:.0f} TF/s", flush=True)
    del a,b,c,bt
