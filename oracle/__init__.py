"""CPU oracle for the BUZZ decode path -- test infrastructure only; the product never imports it."""
