"""Seeded random shapes for the standalone calls (GEMMs and SpMM with pitches and base offsets that are
not 16-byte friendly, empty operands) and random mini-batch, chunk and halo configurations, each
against numpy / the oracle.  The fixed cases elsewhere use the workloads' shapes; these walk the corners."""
import numpy as np
import pytest
import torch

import synth
from oracle import chunks as ochunks
from oracle import graph as og
from oracle import step as ostep
from tests._cases import TOL_FP32, assert_step_grads_close

pytestmark = pytest.mark.gpu
DEV = "cuda"
KEYS = ("l2g", "rowptr", "col", "colptr", "row", "d_local_in", "d_local_out", "d_global_in")


@pytest.fixture(scope="module")
def g():
    import paper_2602_01872_amd as lib
    lib.load()
    return lib


def rel(a, b):
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-30))


def mat(rows, cols, ld, seed, off=0):
    """[rows x cols] view with pitch ld that starts `off` elements into an allocation filled with NaN."""
    buf = torch.full((rows * ld + off + 8,), float("nan"), device=DEV)
    v = buf[off:off + rows * ld].view(rows, ld) if rows > 0 else buf[off:off].view(0, ld)
    x = synth.normal_matrix(max(rows, 1), cols, seed)[:rows]
    if rows > 0:
        v[:, :cols] = x.to(DEV)
    return buf, v, x


@pytest.mark.parametrize("block", range(3))
def test_random_gemm_and_spmm_calls(g, block):
    rng = np.random.default_rng(77 + block)
    for case in range(50):
        op=["nn","nt","tn","spmm"][rng.integers(0,4)]
        seed=int(rng.integers(1,1<<30))
        if op in("nn","nt","tn"):
            M=int(rng.integers(0,20000)) if rng.random()<0.8 else int(rng.integers(0,200))
            N=int(rng.integers(1,300)); K=int(rng.integers(1,300))
            pa=int(rng.integers(0,6)); pb=int(rng.integers(0,6)); pc=int(rng.integers(0,6))
            oa=int(rng.integers(0,4)) if rng.random()<0.3 else 0
            print(f"[case] block {block} case {case}: gemm_{op} M={M} N={N} K={K} pads={pa},{pb},{pc} off={oa}",flush=True)
            if op=="nn":
                ba,A,Ah=mat(M,K,K+pa,seed,oa); bb,B,Bh=mat(K,N,N+pb,seed+1); bc,Cm,_=mat(M,N,N+pc,seed+2)
                g.grp_gemm_nn(M,N,K,A,K+pa,g.DTYPE_FP32,B,N+pb,Cm,N+pc); torch.cuda.synchronize()
                want=Ah.double().numpy()@Bh.double().numpy(); got=Cm[:,:N].cpu().numpy()
            elif op=="nt":
                ba,A,Ah=mat(M,K,K+pa,seed,oa); bb,B,Bh=mat(N,K,K+pb,seed+1); bc,Cm,_=mat(M,N,N+pc,seed+2)
                g.grp_gemm_nt(M,N,K,A,K+pa,g.DTYPE_FP32,B,K+pb,Cm,N+pc); torch.cuda.synchronize()
                want=Ah.double().numpy()@Bh.double().numpy().T; got=Cm[:,:N].cpu().numpy()
            else:
                ba,A,Ah=mat(M,K,K+pa,seed,oa); bb,B,Bh=mat(M,N,N+pb,seed+1); bc,Cm,_=mat(K,N,N+pc,seed+2)
                ws=torch.empty(max(g.grp_gemm_tn_workspace_bytes(M,K,N),16),dtype=torch.uint8,device=DEV)
                g.grp_gemm_tn(M,K,N,A,K+pa,g.DTYPE_FP32,B,N+pb,Cm,N+pc,ws); torch.cuda.synchronize()
                want=Ah.double().numpy().T@Bh.double().numpy(); got=Cm[:,:N].cpu().numpy()
            if want.size and M>0: assert rel(got,want)<=1e-4,(rel(got,want))
            elif want.size: assert (got==0).all()
            # nothing outside the N columns of C was written (pads keep their NaN) unless documented otherwise
        else:
            N=int(rng.integers(10,5000)); E=int(rng.integers(0,50*N)); F=int(rng.integers(1,300)); px=int(rng.integers(0,6)); py=int(rng.integers(0,6))
            tr=bool(rng.integers(0,2)); sc=int(rng.integers(0,3)); st=bool(rng.integers(0,2))
            print(f"[case] block {block} case {case}: spmm N={N} E={E} F={F} pads={px},{py} transposed={tr} scale={sc} self={st}",flush=True)
            s,d=synth.rmat_graph(int(np.ceil(np.log2(N))),E,seed=seed,n_nodes=N)
            part=g.grp_partition(s.to(DEV),d.to(DEV),N,1,1,0)
            bx,X,Xh=mat(N,F,F+px,seed); by,Y,_=mat(N,F,F+py,seed+1)
            g.grp_spmm(part,tr,sc,st,F,X,F+px,g.DTYPE_FP32,Y,F+py); torch.cuda.synchronize()
            a,b=(d,s) if tr else (s,d)          # row owner b gathers a
            xh=Xh.double()
            acc=torch.zeros(N,F,dtype=torch.float64).index_add_(0,b,xh[a])
            deg=torch.bincount(b,minlength=N).double()
            if st: acc+=xh
            if sc==1: acc=acc/torch.clamp(deg,min=1)[:,None]
            elif sc==2: acc=acc/torch.sqrt(torch.clamp(deg+(1 if st else 0),min=1))[:,None]
            got=Y[:,:F].cpu().double().numpy()
            assert rel(got,acc.numpy())<=1e-4,rel(got,acc.numpy())
            part.destroy()


@pytest.mark.parametrize("block", range(3))
def test_random_minibatch_chunk_and_halo_configurations(g, block):
    rng = np.random.default_rng(177 + block)
    for case in range(40):
        kind=["uniform","rmat"][rng.integers(0,2)]
        N=int(rng.integers(20,8000)); E=int(rng.integers(0,60*N)); seed=int(rng.integers(1,1<<30))
        if kind=="rmat":
            s,d=synth.rmat_graph(int(np.ceil(np.log2(N))),E,seed=seed,n_nodes=N)
        else:
            s,d=synth.uniform_graph(N,E,seed=seed)
        sd,dd=s.to(DEV),d.to(DEV)
        mode=["mb","chunks","halo"][rng.integers(0,3)]
        if mode=="chunks":
            c=int(rng.integers(1,9)); b=int(rng.integers(0,c)); w=int(rng.integers(0,c))
            print(f"[case] block {block} case {case}: chunks {kind} N={N} E={E} c={c} base={b} swept={w}",flush=True)
            ck=g.grp_chunks_build(sd,dd,N,c,seed)
            part=g.grp_partition_from_chunks(ck,b,w)
            want=ochunks.partition_from_chunks(s.numpy(),d.numpy(),N,c,seed,b,w)
            for k in KEYS: assert np.array_equal(part.array(k),want[k]),k
            assert np.array_equal(part.base_mask(),want["base_mask"])
            part.destroy(); ck.destroy(); continue
        K=int(rng.integers(1,5)); p=int(rng.integers(0,K))
        if mode=="halo":
            hops=int(rng.integers(1,4))
            print(f"[case] block {block} case {case}: halo {kind} N={N} E={E} K={K} p={p} hops={hops}",flush=True)
            part=g.grp_partition_halo(sd,dd,N,K,seed,p,hops)
            want=og.partition_halo(s.numpy(),d.numpy(),N,K,seed,p,hops)
            for k in KEYS: assert np.array_equal(part.array(k),want[k]),k
            assert np.array_equal(part.base_mask(),want["owned_mask"])
            part.destroy(); continue
        part=g.grp_partition(sd,dd,N,K,seed,p); op=og.partition(s.numpy(),d.numpy(),N,K,seed,p)
        n=part.n
        if n<2: part.destroy(); continue
        k=int(rng.integers(1,4)); dims=[int(rng.integers(1,100)) for _ in range(k+1)]; dims[-1]=int(rng.integers(2,40))
        fan=tuple(int(rng.integers(1,65)) if rng.random()<0.2 else int(rng.integers(1,12)) for _ in range(k))
        ns=int(rng.integers(1,min(n,600)+1))
        seeds=np.sort(rng.choice(n,ns,replace=False)).astype(np.int32) if rng.random()<0.5 else rng.permutation(n)[:ns].astype(np.int32)
        bf16=rng.random()<0.3; est=int(rng.integers(0,4)); batch=int(rng.integers(0,1000))
        print(f"[case] block {block} case {case}: mb {kind} N={N} E={E} K={K} p={p} n={n} dims={dims} fan={fan} seeds={ns} bf16={bf16} est={est}",flush=True)
        x=synth.normal_matrix(n,dims[0],seed)
        if bf16: x=synth.to_bf16_rne(x)
        y=synth.labels(n,dims[-1],seed); theta=synth.model_weights("sage",dims,seed)
        model=g.model_desc(0,dims,g.DTYPE_BF16 if bf16 else g.DTYPE_FP32)
        sdv=torch.from_numpy(seeds).to(DEV)
        opts=g.step_opts(estimator=est,full_graph=False,seeds=sdv,fanouts=fan,sampler_seed=seed,batch_id=batch)
        P=g.grp_param_count(model)
        ws=torch.empty(g.grp_step_workspace_bytes(part,model,opts),dtype=torch.uint8,device=DEV)
        grad=torch.full((P,),float("nan"),device=DEV); stats=g.new_stats(1)
        g.grp_train_step(part,model,opts,x.to(DEV),y.to(DEV),None,theta.to(DEV),ws,grad,stats)
        torch.cuda.synchronize()
        mb=dict(seeds=seeds,fanouts=fan,sampler_seed=seed,batch_id=batch)
        def oracle_fn(relu_flip=None,near_kink=None):
            return ostep.train_step(op,"sage",dims,theta.double().numpy(),x.double().numpy(),y.numpy(),estimator=est,minibatch=mb,relu_flip=relu_flip,near_kink=near_kink)
        gr=grad.cpu().numpy(); assert np.isfinite(gr).all()
        _,ost=assert_step_grads_close(gr,oracle_fn,"sage",dims,TOL_FP32)
        st=g.read_stats(stats)[0]
        assert int(st["S"])==ost["S"] and int(st["nnz_used"])==ost["nnz_used"]
        assert abs(float(st["R"])-ost["R"])<=1e-9*max(1.0,abs(ost["R"]))
        assert abs(float(st["sum_ratio"])-ost["sum_ratio"])<=1e-9*max(1.0,ost["sum_ratio"])
        assert abs(float(st["loss"])-ost["loss"])<=TOL_FP32*max(abs(ost["loss"]),1e-30)
        part.destroy()
