"""CPU oracle for the H1B-KV hot path -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

`oracle.cref` wraps the plain-C implementation (h1bkv_oracle.c); `oracle.exact` is a second,
exact-arithmetic rendering of Eq.(2)-(5) for tiny inputs that the pins compare it with.
Nothing under paper_2510_05529_amd/ may import this package.
"""
